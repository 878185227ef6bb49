// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stddef.h>
#include <string>
#include <vector>

#include "koala.h"

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

enum { KOALA_NSPLIT_MAX = 16, KOALA_TOPK_MAX = 16 };

// Per-row metadata of one pass (verify, draft catch-up, or one draft tree level).
// Row r of the pass belongs to sequence row_b[r]; its key/value go to cache slot
// row_slot[r]; it has rotary position row_pos[r]; it attends to cache slots
// [0, row_nvis[r]) and to slot row_base[r] + j for every set bit j of row_mask[r].
struct RowMeta {
    int32_t *row_b, *row_pos, *row_slot, *row_nvis, *row_base;
    uint64_t *row_mask;
    int32_t *kv_end;   // [batch]: one past the last slot any row of the sequence may see
    float *rope_cos, *rope_sin;  // [rows][head_dim/2]
};

// Device tables describing the static tree (uploaded at bind).
struct TreeTables {
    int32_t *parent, *depth, *rank;   // [T]
    uint64_t *anc_mask;               // [T] bit j: j is the node or one of its ancestors
    int32_t *exp_index;               // [T] index among expanded non-root nodes, or -1
    uint64_t *draft_mask;             // [T] bit e: expanded non-root ancestor-or-self with index e
    int32_t *level_nodes;             // [D][64] expanded nodes of each depth (-1 padded)
    int32_t *child_first, *child_count;  // unused by kernels that scan; kept for clarity
};

struct koala_ctx {
    koala_shape shape;
    koala_draft_shape draft;
    int T, D, max_batch, max_rows;  // max_rows = max_batch * max(T, max_m)
    std::vector<int32_t> parent, rank, topk, depth, exp_index;
    std::vector<uint64_t> anc_mask, draft_mask;
    std::vector<std::vector<int32_t>> level_exp;  // expanded nodes per depth
    int n_exp;                                    // expanded non-root nodes
    std::string err;

    bool bound;
    koala_weights w;
    std::vector<const void *> layer_w, draft_w;
    koala_kv kv;
    char *ws;
    size_t ws_bytes;

    // workspace carve-up (device pointers)
    TreeTables tt;
    RowMeta meta;
    float *x, *act, *qkv, *qrot, *attn_out, *gu, *o_part, *ml, *logits, *fhat, *topk_val;
    int32_t *topk_idx, *tok_tmp;
    // generation loop state of sequence 0 (koala_generate)
    float *gen_dlogits, *gen_tlogits;                    // [T][V] draft / target logits of the non-greedy loop
    float *gen_feat, *gen_feat_in;                       // [T][H] verify features; [max(D+1, max_m)][H] next draft inputs
    int32_t *gen_tree, *gen_greedy, *gen_acc, *gen_path, *gen_next, *gen_tok_in;
    int n_cu;                      // compute units of the device the context is bound on
    int attn_ns;                   // key splits of the attention kernels (fixed at create)
    float *med_logits;                                   // [D * max_batch][V] per-depth logits of Medusa-style heads (sampled drafting)
    float *acc_q, *acc_d;                                // [max_batch][V] distributions of the stochastic acceptance walk
    // bf16 path: GEMM input as fp16 MFMA fragments, and the split-K partial sums
    void *xf, *xf2;   // xf2: input of the down projection (written by the gate/up projection's epilogue)
    float *part;
    size_t xf_bytes, part_bytes;
    void *qf;          // query fragments of the bf16 attention (in the buffer of qrot)
    int *attn_cnt;     // arrival counters of the attention kernel's split merge
    size_t opart_bytes, ml_bytes;
    float *cand_val;   // [rows][ceil(V/1024)][16] top-k candidates of the LM-head epilogue
    int *cand_idx;
    float *row_sums;   // [64 chunks][rows] sums of squares per 512-column chunk (RMSNorm row scale)
    int pend_S, pend_ld, pend_mode;  // partial sums waiting to be folded into x (0 = none)

    // optional event timing of the GEMM launches (koala_profile_begin / _end)
    std::vector<hipEvent_t> prof_ev;
    int prof_used;
    double prof_bytes;
    bool prof_on;
};

#define KOALA_CHECK_LAUNCH(ctx)                                              \
    do {                                                                     \
        hipError_t e__ = hipGetLastError();                                  \
        if (e__ != hipSuccess) {                                             \
            (ctx)->err = std::string("kernel launch failed: ") + hipGetErrorString(e__); \
            return KOALA_E_DEVICE;                                           \
        }                                                                    \
    } while (0)

// ---------------------------------------------------------------------------------------------
// launchers implemented in kernels_generic.hip (is_bf16 selects the storage type of weights/KV)
// ---------------------------------------------------------------------------------------------
namespace kg {

void setup_verify(hipStream_t s, const koala_ctx *c, int batch);
void setup_catchup(hipStream_t s, const koala_ctx *c, int batch, int m);
void setup_level(hipStream_t s, const koala_ctx *c, int batch, int d, int n_level);

void embed_rows(hipStream_t s, bool bf16, const int32_t *tok, const void *E, float *x, int rows, int H);
void fc_input(hipStream_t s, bool bf16, const int32_t *tok, const void *E, const float *feat,
              float *act, int rows, int H);
void rmsnorm(hipStream_t s, bool bf16, const float *x, const void *g, float *out, int rows, int H, float eps);
// Y[M,N] (ldy) = or += A[M,K] (lda) * W[N,K]^T
void gemm(hipStream_t s, bool bf16, const float *A, int lda, const void *W, float *Y, int ldy,
          int M, int N, int K, bool accumulate);
void rope_append(hipStream_t s, bool bf16, const float *qkv, const RowMeta &meta, float *qrot,
                 void *kcache, void *vcache, int rows, int H, int n_heads, int head_dim,
                 int capacity, int max_batch_stride_rows);
void attention(hipStream_t s, bool bf16, const float *qrot, const RowMeta &meta, const void *kcache,
               const void *vcache, float *o_part, float *ml, float *attn_out, int batch,
               int rows_per_seq, int n_heads, int head_dim, int capacity, int nsplit);  // attn_out NULL: no merge
void silu_mul(hipStream_t s, const float *gu, float *act, int rows, int F);
void resblock_update(hipStream_t s, float *x, const float *y, int n);
void topk_rows(hipStream_t s, const float *logits, int ld, int rows, int V, int k, int32_t *idx, float *val);
void copy_f32(hipStream_t s, float *dst, const float *src, size_t n);

// draft bookkeeping
void gather_last_rows(hipStream_t s, const float *x, float *dst, size_t dst_stride, int batch, int m, int H);
void store_fhat(hipStream_t s, const float *x, float *fhat, const int32_t *level_nodes, int batch,
                int n_level, int T, int H);
void level_inputs(hipStream_t s, bool bf16, const int32_t *tree_tokens, const void *E, const float *fhat,
                  const int32_t *level_nodes, const int32_t *parent, float *act, int batch,
                  int n_level, int T, int H);
void set_root(hipStream_t s, const int32_t *tok_in, int m, int32_t *tree_tokens, float *scores, int batch, int T);
void fill_children(hipStream_t s, const int32_t *topk_idx, const float *topk_val, int kmax,
                   const int32_t *level_nodes, int n_level, const TreeTables &tt, int d,
                   int32_t *tree_tokens, float *scores, int batch, int T);
void fill_medusa(hipStream_t s, const int32_t *topk_idx, const float *topk_val, int kmax,
                 const TreeTables &tt, int32_t *tree_tokens, float *scores, int batch, int T, int heads);

void accept_scan(hipStream_t s, const TreeTables &tt, int T, int D, const int32_t *tree_tokens,
                 const int32_t *greedy, int32_t *accept_len, int32_t *accept_path, int32_t *next_token,
                 int batch);
void kv_commit(hipStream_t s, bool bf16, void *kcache, void *vcache, const int32_t *ctx_len,
               const int32_t *accept_len, const int32_t *accept_path, int D, int n_layers,
               int max_batch, int batch, int n_heads, int capacity, int head_dim);
void advance_ctx(hipStream_t s, int32_t *ctx_len, const int32_t *accept_len, int batch);
// measurement aid: read `bytes` (multiple of 16) once with streaming loads
void stream_read(hipStream_t s, const void *src, size_t bytes, unsigned *sink);
// generation loop: next draft inputs (rows 0..a) and emitted tokens from the accepted path of sequence 0
void gen_next(hipStream_t s, const float *feat_out, const int32_t *tree_tokens, const int32_t *accept_len,
              const int32_t *accept_path, const int32_t *next_token, int T, int D, int H, float *feat_next,
              int32_t *tok_next, int32_t *out_tokens, int n_done, int max_new);

}  // namespace kg

// ---------------------------------------------------------------------------------------------
// launchers implemented in kernels_sampling.hip (non-greedy drafting and acceptance, section 2.2)
// ---------------------------------------------------------------------------------------------
namespace ks {

int max_vocab();   // largest vocabulary the sampling kernels handle

// logits: [batch * n_level][V] draft logits of the level's nodes (overwritten); children of those nodes get
// draws without replacement from softmax(logits / temperature); the logits are copied to draft_logits[b][node]
void sample_children(hipStream_t st, float *logits, const int32_t *level_nodes, int n_level, const TreeTables &tt,
                     int T, int V, float temperature, const float *u_draw, int32_t *tree_tokens,
                     float *draft_logits, int batch);
// dst[b * n_level + li][:] = src[src_row0 + b][:] for all li < n_level
void repeat_rows(hipStream_t st, const float *src, int src_row0, float *dst, int V, int n_level, int batch);
void accept_sample(hipStream_t st, const TreeTables &tt, int T, int D, int V, float temperature,
                   const int32_t *tree_tokens, const float *target_logits, const float *draft_logits,
                   const float *u_accept, const float *u_resample, float *qv, float *dv, int32_t *accept_len,
                   int32_t *accept_path, int32_t *next_token, int batch);

}  // namespace ks

// ---------------------------------------------------------------------------------------------
// launchers implemented in kernels_bf16.hip (fragment-major weights and activations in fp16)
// ---------------------------------------------------------------------------------------------
namespace kb {

// number of 16-row activation tiles used for `rows` rows: 1, 2 or a multiple of 4
inline int mt_of(int rows) { return rows <= 16 ? 1 : rows <= 32 ? 2 : 4 * ((rows + 63) / 64); }
inline int pad64(int n) { return (n + 63) / 64 * 64; }

inline size_t xf_bytes(int K, int MT) { return (size_t)(K / 32) * MT * 1024; }
// a packed bf16 weight matrix of n_elements values (a multiple of 8) to the fp16 the GEMMs multiply with, in place
void weights_to_f16(hipStream_t st, void *w, size_t n_elements);

// Pending RMSNorm row scale: 1/sqrt(sum_c sums[c][row] / K + eps); sums == nullptr means scale 1.
struct NormScale {
    const float *sums;
    int nparts, srows, K;
    float eps;
};

int gemm_splits(int Npad, int K, int MTT = 0);
int rows_splits(int Npad, int K);              // split count of gemm_rows_partial   // MTT: activation tiles of the call (0: at most four)
// P[S][MTT*16][Npad] = partial sums of X * W^T, X given as fp16 fragments [K/32][MTT][64] x 16 B
// ev_start/ev_stop (either may be null) are attached to the dispatch: they take the kernel's own begin and end times
void gemm_packed(hipStream_t st, const void *Wp, const void *Xf, float *P, int Npad, int K, int MTT, int S,
                 hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
// Row-group GEMM (one workgroup per few 16-row groups of the weights and K range, waves take 64-k tiles in
// turn; n_cu = compute units of the device, which sets the groups per workgroup), MTT = 1, 2 or 4:
// _partial: P[S][MTT*16][Npad] partial sums, like gemm_packed;  _qkv (S = 1): row scale, rotary embedding,
// queries as attention fragments qf, keys/values into their cache slots (W_q, W_k rows pair-interleaved);  _swiglu (S = 1): row
// scale, SiLU(gate) * up as fragments Xo of the down projection's input
void gemm_rows_partial(hipStream_t st, const void *Wp, const void *Xf, float *P, int Npad, int K, int MTT, int S,
                       hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
void gemm_rows_qkv(hipStream_t st, const void *Wp, const void *Xf, int K, int MTT, const NormScale &ns, int rows,
                   int rows_per_seq, const RowMeta &meta, void *qf, void *kc, void *vc, int H, int n_heads, int head_dim,
                   int cap, int n_cu, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
void gemm_rows_swiglu(hipStream_t st, const void *Wp, const void *Xf, int K, int MTT, const NormScale &ns, int rows,
                      void *Xo, int F, int n_cu, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
// GEMM for many activation rows (MTT >= 8 tiles): P[S][MTT*16][Npad] partial sums; big_shape picks the launch
struct BigShape { int n_mt, n_pm, mtw, U, S; };
BigShape big_shape(int Npad, int K, int rows, int n_cu, bool one_split = false);
void gemm_big(hipStream_t st, const void *Wp, const void *Xf, float *P, int Npad, int K, int MTT, const BigShape &b,
              hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
void gemm_big_qkv(hipStream_t st, const void *Wp, const void *Xf, int K, int MTT, const BigShape &b, const NormScale &ns,
                  int rows, int rows_per_seq, const RowMeta &meta, void *qf, void *kc, void *vc, int H, int n_heads,
                  int head_dim, int cap, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
void gemm_big_swiglu(hipStream_t st, const void *Wp, const void *Xf, int K, int MTT, const BigShape &b,
                     const NormScale &ns, int rows, void *Xo, int F, hipEvent_t ev_start = nullptr,
                     hipEvent_t ev_stop = nullptr);
// v = (mode 1: x +) sum of partials (mode 0: x as is); x <- v for modes 1, 2; Xf (may be NULL) receives the
// fragments of gain * v (gain NULL: v); sums (may be NULL) the sums of squares of v per 512-column chunk
void fold(hipStream_t st, float *x, int ldx, const float *P, int S, int Mp, int ldp, int mode, int M, int N,
          const void *gain, void *Xf, int MT, float *sums, int srows);
// qf: query fragments [batch][n_heads][ceil(rows_per_seq/16)][head_dim/32][hi, lo][64 lanes] x 16 B, times
// 1/sqrt(head_dim)
void rope_append(hipStream_t st, const float *P, int S, int Mp, int ldp, const NormScale &ns, const RowMeta &meta,
                 void *qf, void *kc, void *vc, int rows, int H, int n_heads, int head_dim, int cap, int rows_per_seq);
// tree-masked attention over the cache, key splits merged in the kernel, rows written as fragments Xf of the
// O projection's input; counters: max_batch * n_heads * 4 ints, zero before the first launch
void attention_tree(hipStream_t st, const void *qf, const RowMeta &meta, const void *kc, const void *vc, float *o_part,
                    size_t opart_bytes, float *ml, size_t ml_bytes, int *counters, void *Xf, int MT_out, int batch,
                    int rows_per_seq, int n_heads, int head_dim, int cap, int nsplit);
void silu_frag(hipStream_t st, const float *P, int S, int Mp, int ldp, const NormScale &ns, void *Xf, int MT, int M,
               int F);
void resblock_p(hipStream_t st, float *x, int ldx, const float *P, int S, int Mp, int ldp, int M, int H);
void reduce_out(hipStream_t st, const float *P, int S, int Mp, int ldp, float *out, int ldo, int M, int N);
void logits_topk(hipStream_t st, const float *P, int S, int Mp, int ldp, const NormScale &ns, float *logits, int ldl,
                 int rows, int V, int k, float *cand_val, int *cand_idx, int32_t *idx, float *val);

}  // namespace kb
