// C ABI of the draft-then-verify library: argument validation, workspace layout and the
// sequence of kernel launches for each entry point.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>

#include <mutex>

#include "koala_internal.h"

// Scratch of koala_accept_sample_static: the two distributions of the stochastic acceptance walk,
// [2][KOALA_STATIC_SCRATCH_FLOATS / 2] floats.  Every device the library runs on holds its own copy of
// the array until the process ends.  In host code the array's name is only a handle: the device
// address is looked up once per device (static_scratch) and that pointer is what kernels receive.
enum { KOALA_STATIC_SCRATCH_FLOATS = 2 * 262144 };
static __device__ __align__(256) float scratch[KOALA_STATIC_SCRATCH_FLOATS];

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

koala_status fail(koala_ctx *c, koala_status st, const char *msg) {
    if (c) c->err = msg;
    return st;
}

inline bool aligned16(const void *p) { return (((uintptr_t)p) & 15u) == 0; }

// Walks the workspace; with base == nullptr it only measures.
struct Carver {
    char *base;
    size_t off;
    template <typename T>
    T *take(size_t n) {
        T *p = base ? (T *)(base + off) : nullptr;
        off += up(n * sizeof(T));
        return p;
    }
};

// Device address of `scratch` on the current device, looked up on first use per device.
hipError_t static_scratch(float **out) {
    enum { MAX_DEVICES = 64 };
    static float *ptr[MAX_DEVICES] = {nullptr};
    static std::mutex mu;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = (float *)p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

// Key splits per (head, sequence) of the attention kernels: enough workgroups to cover the chip.  Read once,
// at koala_create (KOALA_ATTN_WGS overrides the target); the workspace is carved for this count.
int attn_nsplit(const koala_shape &s) {
    int target = 256;
    if (const char *e = getenv("KOALA_ATTN_WGS")) target = atoi(e) > 0 ? atoi(e) : target;
    const int ns = target / std::max(1, s.n_heads);
    return std::max(1, std::min((int)KOALA_NSPLIT_MAX, ns));
}

size_t carve(koala_ctx *c, char *base) {
    Carver w{base, 0};
    const koala_shape &s = c->shape;
    const int T = c->T, D = c->D, R = c->max_rows, H = s.hidden, F = s.ffn, V = s.vocab;
    const int half = s.head_dim / 2, ns = c->attn_ns;
    (void)w.take<double>(half);  // inv_freq, first in the workspace
    c->tt.parent = w.take<int32_t>(T);
    c->tt.depth = w.take<int32_t>(T);
    c->tt.rank = w.take<int32_t>(T);
    c->tt.anc_mask = w.take<uint64_t>(T);
    c->tt.exp_index = w.take<int32_t>(T);
    c->tt.draft_mask = w.take<uint64_t>(T);
    c->tt.level_nodes = w.take<int32_t>((size_t)(D + 1) * 64);
    c->tt.child_first = nullptr;
    c->tt.child_count = nullptr;
    c->meta.row_b = w.take<int32_t>(R);
    c->meta.row_pos = w.take<int32_t>(R);
    c->meta.row_slot = w.take<int32_t>(R);
    c->meta.row_nvis = w.take<int32_t>(R);
    c->meta.row_base = w.take<int32_t>(R);
    c->meta.row_mask = w.take<uint64_t>(R);
    c->meta.kv_end = w.take<int32_t>(c->max_batch);
    c->meta.rope_cos = w.take<float>((size_t)R * half);
    c->meta.rope_sin = w.take<float>((size_t)R * half);
    c->x = w.take<float>((size_t)R * H);
    c->act = w.take<float>((size_t)R * std::max(2 * H, F));
    c->qkv = w.take<float>((size_t)R * 3 * H);
    // also holds the bf16 path's query fragments, whose rows are padded to 16 per sequence
    c->qrot = w.take<float>((size_t)c->max_batch * ((R / c->max_batch + 15) / 16 * 16) * H);
    c->qf = c->qrot;
    c->attn_out = w.take<float>((size_t)R * H);
    c->gu = w.take<float>((size_t)R * 2 * F);
    c->o_part = w.take<float>((size_t)R * H * ns);
    c->ml = w.take<float>((size_t)R * s.n_heads * ns * 2);
    c->opart_bytes = (size_t)R * H * ns * sizeof(float);
    c->ml_bytes = (size_t)R * s.n_heads * ns * 2 * sizeof(float);
    c->attn_cnt = w.take<int>((size_t)c->max_batch * s.n_heads * 4);
    c->logits = w.take<float>((size_t)R * V);
    c->fhat = w.take<float>((size_t)c->max_batch * T * H);
    c->topk_val = w.take<float>((size_t)R * KOALA_TOPK_MAX);
    c->topk_idx = w.take<int32_t>((size_t)R * KOALA_TOPK_MAX);
    c->tok_tmp = w.take<int32_t>(R);
    {
        const int gm = std::max(D + 1, c->draft.max_m);
        c->gen_feat = w.take<float>((size_t)T * H);
        c->gen_feat_in = w.take<float>((size_t)gm * H);
        c->gen_tree = w.take<int32_t>(T);
        c->gen_greedy = w.take<int32_t>(T);
        c->gen_acc = w.take<int32_t>(1);
        c->gen_path = w.take<int32_t>(D + 1);
        c->gen_next = w.take<int32_t>(1);
        c->gen_tok_in = w.take<int32_t>(gm);
    }
    c->gen_dlogits = w.take<float>((size_t)T * V);
    c->gen_tlogits = w.take<float>((size_t)T * V);
    c->med_logits = c->draft.kind == KOALA_DRAFT_MEDUSA ? w.take<float>((size_t)D * c->max_batch * V) : nullptr;
    c->acc_q = w.take<float>((size_t)c->max_batch * V);
    c->acc_d = w.take<float>((size_t)c->max_batch * V);
    c->xf = c->xf2 = nullptr;
    c->part = nullptr;
    c->xf_bytes = c->part_bytes = 0;
    if (s.dtype == KOALA_BF16) {
        const int MTmax = kb::mt_of(R);
        const int shapes[6][2] = {{3 * H, H}, {H, H}, {2 * F, H}, {H, F}, {kb::pad64(V), H}, {H, 2 * H}};
        size_t worst = 0;
        for (auto &sh : shapes) {
            const int Np = kb::pad64(sh[0]);
            const int S = std::max(std::max(std::max(kb::gemm_splits(Np, sh[1]), kb::gemm_splits(Np, sh[1], MTmax)),
                                            kb::rows_splits(Np, sh[1])), MTmax >= 8 ? 4 : 1);
            worst = std::max(worst, (size_t)S * Np);
        }
        c->part_bytes = worst * MTmax * 16 * sizeof(float);
        c->xf_bytes = kb::xf_bytes(std::max(2 * H, F), MTmax);
        c->xf = w.take<char>(c->xf_bytes);
        c->xf2 = w.take<char>(kb::xf_bytes(F, MTmax));
        c->part = w.take<float>(c->part_bytes / sizeof(float));
        c->row_sums = w.take<float>((size_t)R * 64);
        c->cand_val = w.take<float>((size_t)R * ((V + 1023) / 1024) * KOALA_TOPK_MAX);
        c->cand_idx = w.take<int>((size_t)R * ((V + 1023) / 1024) * KOALA_TOPK_MAX);
    }
    return w.off;
}

template <typename T>
hipError_t upload(T *dst, const std::vector<T> &src) {
    return hipMemcpy(dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
}

// One Llama decoder layer over `rows` rows (rows_per_seq per sequence) whose metadata is in c->meta.
// lw: in_norm, wqkv, wo, post_norm, wgu, wdown.  x (c->x) is updated in place.
void decoder_layer(koala_ctx *c, hipStream_t st, int batch, int rows_per_seq, const void *const *lw,
                   void *kc, void *vc) {
    const koala_shape &s = c->shape;
    const bool bf = s.dtype == KOALA_BF16;
    const int rows = batch * rows_per_seq, H = s.hidden, F = s.ffn;
    kg::rmsnorm(st, bf, c->x, lw[0], c->act, rows, H, s.rms_eps);
    kg::gemm(st, bf, c->act, H, lw[1], c->qkv, 3 * H, rows, 3 * H, H, false);
    kg::rope_append(st, bf, c->qkv, c->meta, c->qrot, kc, vc, rows, H, s.n_heads, s.head_dim, c->kv.capacity, 0);
    kg::attention(st, bf, c->qrot, c->meta, kc, vc, c->o_part, c->ml, c->attn_out, batch, rows_per_seq, s.n_heads,
                  s.head_dim, c->kv.capacity, c->attn_ns);
    kg::gemm(st, bf, c->attn_out, H, lw[2], c->x, H, rows, H, H, true);
    kg::rmsnorm(st, bf, c->x, lw[3], c->act, rows, H, s.rms_eps);
    kg::gemm(st, bf, c->act, H, lw[4], c->gu, 2 * F, rows, 2 * F, H, false);
    kg::silu_mul(st, c->gu, c->act, rows, F);
    kg::gemm(st, bf, c->act, F, lw[5], c->x, H, rows, H, F, true);
}

// Event pair for the next weight-streaming launch while profiling is on (else nulls); counts its weight bytes.
struct LaunchEvents { hipEvent_t start, stop; };
LaunchEvents timed_launch(koala_ctx *c, double weight_bytes) {
    if (!c->prof_on || (size_t)(c->prof_used + 2) > c->prof_ev.size()) return LaunchEvents{nullptr, nullptr};
    const LaunchEvents ev{c->prof_ev[c->prof_used], c->prof_ev[c->prof_used + 1]};
    c->prof_used += 2;
    c->prof_bytes += weight_bytes;
    return ev;
}

// KOALA_GEMM_BIG=0 (tuning aid, read once): batches of more than 64 rows take the passes of the skinny kernel
bool big_gemm_enabled() {
    static const bool on = !(getenv("KOALA_GEMM_BIG") && atoi(getenv("KOALA_GEMM_BIG")) == 0);
    return on;
}

// the many-row GEMM addresses both operands with 32-bit byte offsets
bool big_fits32(int Npad, int K, int MT) {
    return (double)Npad * K * 2.0 < 4.0e9 && (double)(K / 32) * MT * 1024.0 < 4.0e9;
}

// Split-K GEMM on the fragments in Xf (default: c->xf): partial sums of X * W^T into c->part; returns the split count.
int bf_gemm(koala_ctx *c, hipStream_t st, const void *Wp, int N, int K, int MT, int rows = 0, const void *Xf = nullptr) {
    const int Npad = kb::pad64(N);
    if (!Xf) Xf = c->xf;
    const LaunchEvents ev = timed_launch(c, (double)Npad * K * 2.0);
    // many rows: one pass over the weights with large register tiles
    if (MT >= 8 && big_fits32(Npad, K, MT) && big_gemm_enabled()) {
        const kb::BigShape b = kb::big_shape(Npad, K, rows > 0 ? rows : MT * 16, c->n_cu);
        kb::gemm_big(st, Wp, Xf, c->part, Npad, K, MT, b, ev.start, ev.stop);
        return b.S;
    }
    const int S = kb::gemm_splits(Npad, K, MT);
    kb::gemm_packed(st, Wp, Xf, c->part, Npad, K, MT, S, ev.start, ev.stop);
    return S;
}

// Split-K GEMM for at most four activation tiles with the row-group kernel (64 weight rows per workgroup, the
// K range cut so that the launch is about one workgroup per compute unit); fragments from Xf
int bf_gemm_rows(koala_ctx *c, hipStream_t st, const void *Wp, const void *Xf, int N, int K, int MT) {
    const int Npad = kb::pad64(N), S = kb::rows_splits(Npad, K);
    const LaunchEvents ev = timed_launch(c, (double)Npad * K * 2.0);
    kb::gemm_rows_partial(st, Wp, Xf, c->part, Npad, K, MT, S, ev.start, ev.stop);
    return S;
}

kb::NormScale no_scale() { return kb::NormScale{nullptr, 0, 0, 1, 0.f}; }

// row scale of an RMSNorm over the hidden dimension whose chunk sums are in c->row_sums
kb::NormScale hidden_scale(const koala_ctx *c) {
    const int H = c->shape.hidden;
    return kb::NormScale{c->row_sums, (H + 511) / 512, c->max_rows, H, c->shape.rms_eps};
}

// Folds the pending partial sums (of a down projection or of the EAGLE fc; none: x as is) into c->x.
// With `gain` it also leaves gain * x as GEMM fragments and the chunk sums for the row scale.
void fold_pending(koala_ctx *c, hipStream_t st, int rows, int MT, const void *gain) {
    const int H = c->shape.hidden;
    kb::fold(st, c->x, H, c->part, c->pend_S, MT * 16, c->pend_ld, c->pend_S ? c->pend_mode : 0, rows, H, gain,
             gain ? c->xf : nullptr, MT, gain ? c->row_sums : nullptr, c->max_rows);
    c->pend_S = 0;
}

// fp32 rows -> GEMM fragments (no normalisation)
void rows_to_frags(koala_ctx *c, hipStream_t st, const float *a, int lda, int rows, int K, int MT) {
    kb::fold(st, const_cast<float *>(a), lda, nullptr, 0, 0, 0, 0, rows, K, nullptr, c->xf, MT, nullptr, 0);
}

// bf16 decoder layer.  On entry c->pend_* may describe partial sums still to be folded into x; on exit
// the down projection's are pending.  Up to 64 rows: seven launches (fold, QKV projection with rotary embedding
// and cache append, attention, merge of its key splits, O projection, fold, gate/up projection with SwiGLU,
// down projection).  More rows: the projections run in passes with their element-wise steps as kernels of
// their own.
void decoder_layer_bf16(koala_ctx *c, hipStream_t st, int batch, int rows_per_seq, const void *const *lw,
                        void *kc, void *vc) {
    const koala_shape &s = c->shape;
    const int rows = batch * rows_per_seq, H = s.hidden, F = s.ffn, MT = kb::mt_of(rows), Mp = MT * 16;
    // key splits of the attention: as many as keep the launch within one workgroup per compute unit (sequences of
    // more than 32 rows take two workgroups per split and head), at most the count the workspace was carved for
    // and no more than give every one of a workgroup's eight waves one 32-key step of a full cache (more splits
    // only add partial results for the merging workgroup to take in; the context length itself lives on the device)
    const int ns_room = std::max(1, std::min(c->attn_ns, c->n_cu / (s.n_heads * batch * (rows_per_seq > 32 ? 2 : 1))));
    const int ns = std::min(ns_room, std::max(1, ((c->kv.capacity + 31) / 32 + 7) / 8));
    const bool fused = MT <= 4;
    fold_pending(c, st, rows, MT, lw[0]);
    int S;
    if (fused) {
        const LaunchEvents ev = timed_launch(c, 3.0 * H * H * 2.0);
        kb::gemm_rows_qkv(st, lw[1], c->xf, H, MT, hidden_scale(c), rows, rows_per_seq, c->meta, c->qf, kc, vc, H,
                          s.n_heads, s.head_dim, c->kv.capacity, c->n_cu, ev.start, ev.stop);
    } else {
        const int Np = kb::pad64(3 * H);
        if (MT >= 8 && big_fits32(Np, H, MT) && big_gemm_enabled()) {
            // many rows: rotary embedding, KV append and query fragments on the accumulators of the projection
            const LaunchEvents ev = timed_launch(c, (double)Np * H * 2.0);
            const kb::BigShape b = kb::big_shape(Np, H, rows, c->n_cu, true);
            kb::gemm_big_qkv(st, lw[1], c->xf, H, MT, b, hidden_scale(c), rows, rows_per_seq, c->meta, c->qf, kc, vc, H,
                             s.n_heads, s.head_dim, c->kv.capacity, ev.start, ev.stop);
        } else {
            S = bf_gemm(c, st, lw[1], 3 * H, H, MT, rows);
            kb::rope_append(st, c->part, S, Mp, 3 * H, hidden_scale(c), c->meta, c->qf, kc, vc, rows, H, s.n_heads,
                            s.head_dim, c->kv.capacity, rows_per_seq);
        }
    }
    kb::attention_tree(st, c->qf, c->meta, kc, vc, c->o_part, c->opart_bytes, c->ml, c->ml_bytes, c->attn_cnt, c->xf,
                       MT, batch, rows_per_seq, s.n_heads, s.head_dim, c->kv.capacity, ns);
    S = fused ? bf_gemm_rows(c, st, lw[2], c->xf, H, H, MT) : bf_gemm(c, st, lw[2], H, H, MT, rows);
    kb::fold(st, c->x, H, c->part, S, Mp, H, 1, rows, H, lw[3], c->xf, MT, c->row_sums, c->max_rows);
    if (fused) {
        const LaunchEvents ev = timed_launch(c, (double)kb::pad64(2 * F) * H * 2.0);
        kb::gemm_rows_swiglu(st, lw[4], c->xf, H, MT, hidden_scale(c), rows, c->xf2, F, c->n_cu, ev.start, ev.stop);
        S = bf_gemm_rows(c, st, lw[5], c->xf2, H, F, MT);
    } else {
        const int Np = kb::pad64(2 * F);
        if (MT >= 8 && big_fits32(Np, H, MT) && big_gemm_enabled()) {
            // many rows: SwiGLU on the accumulators of the gate/up projection, straight into the down projection's input
            const LaunchEvents ev = timed_launch(c, (double)Np * H * 2.0);
            const kb::BigShape b = kb::big_shape(Np, H, rows, c->n_cu, true);
            kb::gemm_big_swiglu(st, lw[4], c->xf, H, MT, b, hidden_scale(c), rows, c->xf2, F, ev.start, ev.stop);
            S = bf_gemm(c, st, lw[5], H, F, MT, rows, c->xf2);
        } else {
            S = bf_gemm(c, st, lw[4], 2 * F, H, MT, rows);
            kb::silu_frag(st, c->part, S, Mp, 2 * F, hidden_scale(c), c->xf, MT, rows, F);
            S = bf_gemm(c, st, lw[5], H, F, MT, rows);
        }
    }
    c->pend_S = S;
    c->pend_ld = H;
    c->pend_mode = 1;
}

// top-k of the LM-head logits of `rows` fp32 rows at a (row stride lda)
void bf_lm_head_topk(koala_ctx *c, hipStream_t st, const float *a, int lda, int rows, int k, int32_t *idx,
                     float *val) {
    const koala_shape &s = c->shape;
    const int MT = kb::mt_of(rows), Vp = kb::pad64(s.vocab);
    rows_to_frags(c, st, a, lda, rows, s.hidden, MT);
    const int S = bf_gemm(c, st, c->w.lm_head, s.vocab, s.hidden, MT);
    kb::logits_topk(st, c->part, S, MT * 16, Vp, no_scale(), nullptr, 0, rows, s.vocab, k, c->cand_val, c->cand_idx,
                    idx, val);
}

size_t elt(const koala_ctx *c) { return c->shape.dtype == KOALA_BF16 ? 2 : 4; }

size_t layer_stride_bytes(const koala_ctx *c) {
    return (size_t)c->max_batch * c->shape.n_heads * c->kv.capacity * c->shape.head_dim * elt(c);
}

koala_status check_call(koala_ctx *c, int batch) {
    if (!c) return KOALA_E_NULL;
    c->err.clear();
    if (!c->bound) return fail(c, KOALA_E_WORKSPACE, "context is not bound (call koala_bind first)");
    if (batch < 1 || batch > c->max_batch) return fail(c, KOALA_E_SHAPE, "batch must be in 1..max_batch");
    return KOALA_OK;
}

}  // namespace

extern "C" {

koala_status koala_create(const koala_shape *shape, const koala_draft_shape *draft, const koala_tree *tree,
                          int max_batch, koala_ctx **out) {
    if (!shape || !draft || !tree || !out) return KOALA_E_NULL;
    *out = nullptr;
    if (!tree->parent || !tree->rank || (tree->depth > 0 && !tree->topk_per_depth)) return KOALA_E_NULL;
    const koala_shape &s = *shape;
    if (s.hidden <= 0 || s.n_heads <= 0 || s.head_dim <= 0 || s.ffn <= 0 || s.vocab <= 0 || s.n_layers <= 0 ||
        s.hidden != s.n_heads * s.head_dim || max_batch < 1 || s.hidden % 4 || s.ffn % 4 || !(s.rms_eps >= 0.f) ||
        !(s.rope_base > 0.f))
        return KOALA_E_SHAPE;
    if (s.dtype != KOALA_FP32 && s.dtype != KOALA_BF16) return KOALA_E_UNSUPPORTED;
    if (s.head_dim != 64 && s.head_dim != 128) return KOALA_E_UNSUPPORTED;
    if (s.dtype == KOALA_BF16 && (s.hidden % 128 || s.ffn % 128 || s.vocab > 65536)) return KOALA_E_UNSUPPORTED;
    if (draft->kind != KOALA_DRAFT_EAGLE && draft->kind != KOALA_DRAFT_MEDUSA) return KOALA_E_UNSUPPORTED;
    if (draft->K < 1 || draft->max_m < 1 || draft->max_m > KOALA_MAX_M) return KOALA_E_SHAPE;
    const int T = tree->n_nodes, D = tree->depth;
    if (T < 1 || T > KOALA_MAX_NODES || D < 0 || D >= T + (T == 1)) return KOALA_E_SHAPE;
    if (draft->kind == KOALA_DRAFT_MEDUSA && draft->medusa_heads < D) return KOALA_E_SHAPE;

    koala_ctx *c = new koala_ctx();
    c->shape = s;
    c->draft = *draft;
    c->T = T;
    c->D = D;
    c->max_batch = max_batch;
    c->max_rows = max_batch * std::max(std::max(T, draft->max_m), std::max(1, draft->medusa_heads));
    c->bound = false;
    c->ws = nullptr;
    c->prof_on = false;
    c->prof_used = 0;
    c->prof_bytes = 0.0;
    c->pend_S = 0;
    c->attn_ns = attn_nsplit(s);
    c->n_cu = 256;
    c->parent.assign(tree->parent, tree->parent + T);
    c->rank.assign(tree->rank, tree->rank + T);
    c->topk.assign(tree->topk_per_depth, tree->topk_per_depth + D);
    c->depth.assign(T, 0);
    c->anc_mask.assign(T, 0);
    bool ok = c->parent[0] == -1;
    int maxd = 0;
    for (int i = 0; ok && i < T; ++i) {
        if (i > 0) {
            const int p = c->parent[i];
            if (p < 0 || p >= i) { ok = false; break; }
            c->depth[i] = c->depth[p] + 1;
            if (c->depth[i] < c->depth[i - 1]) ok = false;  // nodes ordered by depth
            c->anc_mask[i] = c->anc_mask[p];
            if (c->depth[i] > D) { ok = false; break; }
            const int k = c->topk[c->depth[i] - 1];
            if (c->rank[i] < 0 || c->rank[i] >= k) ok = false;
            for (int j = 1; j < i; ++j)
                if (c->parent[j] == p && c->rank[j] == c->rank[i]) ok = false;
        }
        c->anc_mask[i] |= 1ull << i;
        maxd = std::max(maxd, c->depth[i]);
    }
    for (int d = 0; ok && d < D; ++d)
        if (c->topk[d] < 1 || c->topk[d] > KOALA_TOPK_MAX) ok = false;
    if (!ok || maxd != D) {
        delete c;
        return KOALA_E_SHAPE;
    }
    // nodes with children ("expanded"), per depth; non-root ones get a draft-cache slot index
    std::vector<char> has_child(T, 0);
    for (int i = 1; i < T; ++i) has_child[c->parent[i]] = 1;
    c->exp_index.assign(T, -1);
    c->draft_mask.assign(T, 0);
    c->level_exp.assign(D + 1, {});
    c->n_exp = 0;
    for (int i = 0; i < T; ++i) {
        if (!has_child[i]) continue;
        c->level_exp[c->depth[i]].push_back(i);
        if (i == 0) continue;
        c->exp_index[i] = c->n_exp++;
        c->draft_mask[i] = c->draft_mask[c->parent[i]] | (1ull << c->exp_index[i]);
    }
    *out = c;
    return KOALA_OK;
}

koala_status koala_workspace_bytes(const koala_ctx *ctx, size_t *out) {
    if (!ctx || !out) return KOALA_E_NULL;
    *out = carve(const_cast<koala_ctx *>(ctx), nullptr);
    if (ctx->bound) carve(const_cast<koala_ctx *>(ctx), ctx->ws);  // restore the live pointers
    return KOALA_OK;
}

koala_status koala_bind(koala_ctx *c, const koala_weights *w, const koala_kv *kv, void *workspace, size_t bytes) {
    if (!c) return KOALA_E_NULL;
    c->err.clear();
    if (!w || !kv || !workspace) return fail(c, KOALA_E_NULL, "weights, kv and workspace must not be NULL");
    const bool eagle = c->draft.kind == KOALA_DRAFT_EAGLE;
    if (!w->embed || !w->lm_head || !w->final_norm || !w->layer_w || !w->draft_w || (eagle && !w->fc))
        return fail(c, KOALA_E_NULL, "a weight pointer is NULL");
    if (!kv->target_k || !kv->target_v || !kv->ctx_len || (eagle && (!kv->draft_k || !kv->draft_v)))
        return fail(c, KOALA_E_NULL, "a KV-cache pointer is NULL");
    const int n_lw = 6 * c->shape.n_layers;
    const int n_dw = eagle ? 6 * c->draft.K : c->draft.medusa_heads * c->draft.K;
    for (int i = 0; i < n_lw; ++i)
        if (!w->layer_w[i]) return fail(c, KOALA_E_NULL, "a target layer weight pointer is NULL");
    for (int i = 0; i < n_dw; ++i)
        if (!w->draft_w[i]) return fail(c, KOALA_E_NULL, "a draft weight pointer is NULL");
    bool al = aligned16(w->embed) && aligned16(w->lm_head) && aligned16(w->final_norm) && aligned16(w->fc) &&
              aligned16(kv->target_k) && aligned16(kv->target_v) && aligned16(kv->draft_k) &&
              aligned16(kv->draft_v) && (((uintptr_t)workspace) % ALIGN == 0);
    for (int i = 0; i < n_lw; ++i) al = al && aligned16(w->layer_w[i]);
    for (int i = 0; i < n_dw; ++i) al = al && aligned16(w->draft_w[i]);
    if (!al) return fail(c, KOALA_E_ALIGN, "device pointers must be 16-byte aligned (workspace: 256)");
    if (kv->capacity < c->T + 1) return fail(c, KOALA_E_CAPACITY, "KV capacity smaller than the tree");
    const size_t need = carve(c, nullptr);
    if (bytes < need) {
        if (c->bound) carve(c, c->ws);
        return fail(c, KOALA_E_WORKSPACE, "workspace too small");
    }
    if (c->opart_bytes > 0xFFFFFFF0ull) {
        c->bound = false;
        return fail(c, KOALA_E_UNSUPPORTED, "attention partial results exceed 4 GiB: reduce max_batch");
    }
    c->w = *w;
    c->layer_w.assign(w->layer_w, w->layer_w + n_lw);
    c->draft_w.assign(w->draft_w, w->draft_w + n_dw);
    c->w.layer_w = c->layer_w.data();
    c->w.draft_w = c->draft_w.data();
    c->kv = *kv;
    c->ws = (char *)workspace;
    c->ws_bytes = bytes;
    carve(c, c->ws);

    const int T = c->T, D = c->D, half = c->shape.head_dim / 2;
    std::vector<double> inv_freq(half);
    for (int i = 0; i < half; ++i)
        inv_freq[i] = pow((double)c->shape.rope_base, -2.0 * (double)i / (double)c->shape.head_dim);
    std::vector<int32_t> levels((size_t)(D + 1) * 64, -1);
    for (int d = 0; d <= D; ++d)
        for (size_t i = 0; i < c->level_exp[d].size(); ++i) levels[(size_t)d * 64 + i] = c->level_exp[d][i];
    hipError_t e = hipMemcpy(c->ws, inv_freq.data(), half * sizeof(double), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = upload(c->tt.parent, c->parent);
    if (e == hipSuccess) e = upload(c->tt.depth, c->depth);
    if (e == hipSuccess) e = upload(c->tt.rank, c->rank);
    if (e == hipSuccess) e = upload(c->tt.anc_mask, c->anc_mask);
    if (e == hipSuccess) e = upload(c->tt.exp_index, c->exp_index);
    if (e == hipSuccess) e = upload(c->tt.draft_mask, c->draft_mask);
    if (e == hipSuccess) e = upload(c->tt.level_nodes, levels);
    if (e == hipSuccess) {
        float *unused = nullptr;   // looks up this device's copy of the static scratch array
        e = static_scratch(&unused);
    }
    if (e == hipSuccess) e = hipMemset(c->attn_cnt, 0, (size_t)c->max_batch * c->shape.n_heads * 4 * sizeof(int));
    if (e == hipSuccess) {
        int dev = 0;
        hipDeviceProp_t prop;
        e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
        if (e == hipSuccess) c->n_cu = prop.multiProcessorCount;
    }
    if (e != hipSuccess) {
        c->bound = false;
        c->err = std::string("table upload failed: ") + hipGetErrorString(e);
        return KOALA_E_DEVICE;
    }
    (void)T;
    c->bound = true;
    return KOALA_OK;
}

koala_status koala_tree_verify(koala_ctx *c, void *hip_stream, int batch, const int32_t *tree_tokens,
                               float *feat_out, float *logits_out, int32_t *greedy_out) {
    koala_status st0 = check_call(c, batch);
    if (st0 != KOALA_OK) return st0;
    if (!tree_tokens || !feat_out || !greedy_out) return fail(c, KOALA_E_NULL, "tree_tokens, feat_out, greedy_out required");
    if (!aligned16(tree_tokens) || !aligned16(feat_out) || !aligned16(logits_out) || !aligned16(greedy_out))
        return fail(c, KOALA_E_ALIGN, "device pointers must be 16-byte aligned");
    hipStream_t st = (hipStream_t)hip_stream;
    const koala_shape &s = c->shape;
    const bool bf = s.dtype == KOALA_BF16;
    const int T = c->T, rows = batch * T, H = s.hidden, V = s.vocab;
    kg::setup_verify(st, c, batch);
    kg::embed_rows(st, bf, tree_tokens, c->w.embed, c->x, rows, H);
    const size_t ls = layer_stride_bytes(c);
    float *logits = logits_out ? logits_out : c->logits;
    if (bf) {
        const int MT = kb::mt_of(rows), Mp = MT * 16;
        c->pend_S = 0;
        for (int l = 0; l < s.n_layers; ++l)
            decoder_layer_bf16(c, st, batch, T, c->w.layer_w + 6 * l, (char *)c->kv.target_k + ls * l,
                               (char *)c->kv.target_v + ls * l);
        // last down projection folded in; the LM head runs on gain * x and its logits take the row scale;
        // the features (an output) are normalised separately
        fold_pending(c, st, rows, MT, c->w.final_norm);
        kg::rmsnorm(st, true, c->x, c->w.final_norm, feat_out, rows, H, s.rms_eps);
        const int S = bf_gemm(c, st, c->w.lm_head, V, H, MT);
        kb::logits_topk(st, c->part, S, Mp, kb::pad64(V), hidden_scale(c), logits_out, V, rows, V, 1, c->cand_val,
                        c->cand_idx, greedy_out, nullptr);
        KOALA_CHECK_LAUNCH(c);
        return KOALA_OK;
    }
    for (int l = 0; l < s.n_layers; ++l)
        decoder_layer(c, st, batch, T, c->w.layer_w + 6 * l, (char *)c->kv.target_k + ls * l,
                      (char *)c->kv.target_v + ls * l);
    kg::rmsnorm(st, bf, c->x, c->w.final_norm, feat_out, rows, H, s.rms_eps);
    kg::gemm(st, bf, feat_out, H, c->w.lm_head, logits, V, rows, V, H, false);
    kg::topk_rows(st, logits, V, rows, V, 1, greedy_out, nullptr);
    KOALA_CHECK_LAUNCH(c);
    return KOALA_OK;
}

// u_draw == nullptr: children are the parent's top-k tokens by rank.  Otherwise they are draws without
// replacement from softmax(draft logits / temperature) with the uniforms u_draw[b][child], and the logits of
// every node that has children are stored to draft_logits[b][node][:].
static koala_status draft_expand_impl(koala_ctx *c, void *hip_stream, int batch, const float *feat_in,
                                      const int32_t *tok_in, int m, int32_t *tree_tokens, float *tree_scores,
                                      const float *u_draw, float temperature, float *draft_logits) {
    koala_status st0 = check_call(c, batch);
    if (st0 != KOALA_OK) return st0;
    if (!feat_in || !tok_in || !tree_tokens) return fail(c, KOALA_E_NULL, "feat_in, tok_in, tree_tokens required");
    if (m < 1 || m > c->draft.max_m) return fail(c, KOALA_E_SHAPE, "m must be in 1..max_m");
    if (!aligned16(feat_in) || !aligned16(tok_in) || !aligned16(tree_tokens) || !aligned16(tree_scores) ||
        !aligned16(u_draw) || !aligned16(draft_logits))
        return fail(c, KOALA_E_ALIGN, "device pointers must be 16-byte aligned");
    const bool sampling = u_draw != nullptr;
    if (sampling) {
        if (!draft_logits) return fail(c, KOALA_E_NULL, "draft_logits is required when sampling");
        if (!(temperature > 0.f)) return fail(c, KOALA_E_SHAPE, "temperature must be positive");
        if (c->shape.vocab > ks::max_vocab())
            return fail(c, KOALA_E_UNSUPPORTED, "vocabulary too large for the sampling kernels");
    }
    hipStream_t st = (hipStream_t)hip_stream;
    const koala_shape &s = c->shape;
    const bool bf = s.dtype == KOALA_BF16;
    const int T = c->T, D = c->D, H = s.hidden, V = s.vocab, K = c->draft.K;
    int kmax = 1;
    for (int d = 0; d < D; ++d) kmax = std::max(kmax, c->topk[d]);
    kg::set_root(st, tok_in, m, tree_tokens, tree_scores, batch, T);

    if (c->draft.kind == KOALA_DRAFT_MEDUSA) {
        // head j works on row block j of c->x: rows j*batch .. j*batch + batch - 1
        for (int j = 0; j < D; ++j)
            kg::gather_last_rows(st, feat_in, c->x + (size_t)j * batch * H, (size_t)H, batch, m, H);
        for (int j = 0; j < D; ++j) {
            float *xj = c->x + (size_t)j * batch * H;
            for (int k = 0; k < K; ++k) {
                if (bf) {
                    const int MT = kb::mt_of(batch);
                    rows_to_frags(c, st, xj, H, batch, H, MT);
                    const int S = MT <= 4 ? bf_gemm_rows(c, st, c->w.draft_w[j * K + k], c->xf, H, H, MT)
                                          : bf_gemm(c, st, c->w.draft_w[j * K + k], H, H, MT);
                    kb::resblock_p(st, xj, H, c->part, S, MT * 16, H, batch, H);
                } else {
                    kg::gemm(st, bf, xj, H, c->w.draft_w[j * K + k], c->gu, H, batch, H, H, false);
                    kg::resblock_update(st, xj, c->gu, batch * H);
                }
            }
        }
        if (D > 0 && sampling) {
            // logits of the D heads (row j * batch + b), then per depth one private copy per parent node, from
            // which that node's children are drawn
            if (bf) {
                const int MT = kb::mt_of(D * batch), Vp = kb::pad64(V);
                rows_to_frags(c, st, c->x, H, D * batch, H, MT);
                const int S = bf_gemm(c, st, c->w.lm_head, V, H, MT);
                kb::logits_topk(st, c->part, S, MT * 16, Vp, no_scale(), c->med_logits, V, D * batch, V, 1,
                                c->cand_val, c->cand_idx, c->topk_idx, c->topk_val);
            } else {
                kg::gemm(st, bf, c->x, H, c->w.lm_head, c->med_logits, V, D * batch, V, H, false);
            }
            for (int d = 0; d < D; ++d) {
                const int nl = (int)c->level_exp[d].size();
                if (nl == 0) continue;
                ks::repeat_rows(st, c->med_logits, d * batch, c->logits, V, nl, batch);
                ks::sample_children(st, c->logits, c->tt.level_nodes + (size_t)d * 64, nl, c->tt, T, V, temperature,
                                    u_draw, tree_tokens, draft_logits, batch);
            }
        } else if (D > 0) {
            if (bf) {
                bf_lm_head_topk(c, st, c->x, H, D * batch, kmax, c->topk_idx, c->topk_val);
            } else {
                kg::gemm(st, bf, c->x, H, c->w.lm_head, c->logits, V, D * batch, V, H, false);
                kg::topk_rows(st, c->logits, V, D * batch, V, kmax, c->topk_idx, c->topk_val);
            }
            kg::fill_medusa(st, c->topk_idx, c->topk_val, kmax, c->tt, tree_tokens, tree_scores, batch, T, D);
        }
        KOALA_CHECK_LAUNCH(c);
        return KOALA_OK;
    }

    // EAGLE-style: catch-up rows first, then one pass per tree depth that has expanded nodes
    const size_t ls = layer_stride_bytes(c);
    // fc over [embedding ; feature] then the K draft layers; leaves the predicted features in c->x
    auto run_head = [&](int rows_per_seq) {
        const int rows = batch * rows_per_seq;
        if (bf) {
            const int MT = kb::mt_of(rows), Mp = MT * 16;
            rows_to_frags(c, st, c->act, 2 * H, rows, 2 * H, MT);
            c->pend_S = MT <= 4 ? bf_gemm_rows(c, st, c->w.fc, c->xf, H, 2 * H, MT) : bf_gemm(c, st, c->w.fc, H, 2 * H, MT);
            c->pend_ld = H;
            c->pend_mode = 2;
            for (int k = 0; k < K; ++k)
                decoder_layer_bf16(c, st, batch, rows_per_seq, c->w.draft_w + 6 * k, (char *)c->kv.draft_k + ls * k,
                                   (char *)c->kv.draft_v + ls * k);
            fold_pending(c, st, rows, MT, nullptr);
        } else {
            kg::gemm(st, bf, c->act, 2 * H, c->w.fc, c->x, H, rows, H, 2 * H, false);
            for (int k = 0; k < K; ++k)
                decoder_layer(c, st, batch, rows_per_seq, c->w.draft_w + 6 * k, (char *)c->kv.draft_k + ls * k,
                              (char *)c->kv.draft_v + ls * k);
        }
    };
    // LM head on `rows` fp32 rows at a (row stride lda), then the children of the level's nodes: their
    // parent's top-k tokens by rank, or draws from the parent's distribution
    auto head_children = [&](float *a, int lda, int rows, int d, const int32_t *lv, int nl) {
        const int k = c->topk[d];
        if (bf) {
            const int MT = kb::mt_of(rows), Vp = kb::pad64(V);
            rows_to_frags(c, st, a, lda, rows, H, MT);
            const int S = bf_gemm(c, st, c->w.lm_head, V, H, MT);
            kb::logits_topk(st, c->part, S, MT * 16, Vp, no_scale(), sampling ? c->logits : nullptr, V, rows, V,
                            sampling ? 1 : k, c->cand_val, c->cand_idx, c->topk_idx, c->topk_val);
        } else {
            kg::gemm(st, bf, a, lda, c->w.lm_head, c->logits, V, rows, V, H, false);
            if (!sampling) kg::topk_rows(st, c->logits, V, rows, V, k, c->topk_idx, c->topk_val);
        }
        if (sampling)
            ks::sample_children(st, c->logits, lv, nl, c->tt, T, V, temperature, u_draw, tree_tokens, draft_logits,
                                batch);
        else
            kg::fill_children(st, c->topk_idx, c->topk_val, k, lv, nl, c->tt, d, tree_tokens, tree_scores, batch, T);
    };
    kg::setup_catchup(st, c, batch, m);
    kg::fc_input(st, bf, tok_in, c->w.embed, feat_in, c->act, batch * m, H);
    run_head(m);
    if (D > 0) {
        // root's predicted feature -> fhat[b][0]; its logits decide the depth-1 tokens
        kg::gather_last_rows(st, c->x, c->fhat, (size_t)T * H, batch, m, H);
        head_children(c->fhat, T * H, batch, 0, c->tt.level_nodes, 1);
    }
    for (int d = 1; d < D; ++d) {
        const int nl = (int)c->level_exp[d].size();
        if (nl == 0) continue;
        const int32_t *lv = c->tt.level_nodes + (size_t)d * 64;
        kg::setup_level(st, c, batch, d, nl);
        kg::level_inputs(st, bf, tree_tokens, c->w.embed, c->fhat, lv, c->tt.parent, c->act, batch, nl, T, H);
        run_head(nl);
        kg::store_fhat(st, c->x, c->fhat, lv, batch, nl, T, H);
        head_children(c->x, H, batch * nl, d, lv, nl);
    }
    KOALA_CHECK_LAUNCH(c);
    return KOALA_OK;
}

koala_status koala_draft_expand(koala_ctx *c, void *hip_stream, int batch, const float *feat_in,
                                const int32_t *tok_in, int m, int32_t *tree_tokens, float *tree_scores) {
    return draft_expand_impl(c, hip_stream, batch, feat_in, tok_in, m, tree_tokens, tree_scores, nullptr, 1.f,
                             nullptr);
}

koala_status koala_draft_expand_sample(koala_ctx *c, void *hip_stream, int batch, const float *feat_in,
                                       const int32_t *tok_in, int m, const float *u_draw, float temperature,
                                       int32_t *tree_tokens, float *draft_logits) {
    if (c && !u_draw) return fail(c, KOALA_E_NULL, "u_draw is required");
    return draft_expand_impl(c, hip_stream, batch, feat_in, tok_in, m, tree_tokens, nullptr, u_draw, temperature,
                             draft_logits);
}

static koala_status accept_sample_impl(koala_ctx *c, void *hip_stream, int batch, const int32_t *tree_tokens,
                                       const float *target_logits, const float *draft_logits,
                                       const float *u_accept, const float *u_resample, float temperature,
                                       int32_t *accept_len, int32_t *accept_path, int32_t *next_token, int commit,
                                       bool use_static) {
    koala_status st0 = check_call(c, batch);
    if (st0 != KOALA_OK) return st0;
    if (!tree_tokens || !target_logits || !u_accept || !u_resample || !accept_len || !accept_path || !next_token ||
        (c->T > 1 && !draft_logits))
        return fail(c, KOALA_E_NULL, "all accept_sample pointers are required");
    if (!(temperature > 0.f)) return fail(c, KOALA_E_SHAPE, "temperature must be positive");
    if (c->shape.vocab > ks::max_vocab())
        return fail(c, KOALA_E_UNSUPPORTED, "vocabulary too large for the sampling kernels");
    const koala_shape &s = c->shape;
    float *qv = c->acc_q, *dv = c->acc_d;
    if (use_static) {
        if ((size_t)batch * (size_t)s.vocab > KOALA_STATIC_SCRATCH_FLOATS / 2)
            return fail(c, KOALA_E_CAPACITY, "koala_accept_sample_static: batch * vocab exceeds 262144");
        float *base = nullptr;
        const hipError_t e = static_scratch(&base);
        if (e != hipSuccess) {
            c->err = std::string("static scratch look-up failed: ") + hipGetErrorString(e);
            return KOALA_E_DEVICE;
        }
        qv = base;
        dv = base + KOALA_STATIC_SCRATCH_FLOATS / 2;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    ks::accept_sample(st, c->tt, c->T, c->D, s.vocab, temperature, tree_tokens, target_logits, draft_logits,
                      u_accept, u_resample, qv, dv, accept_len, accept_path, next_token, batch);
    if (commit) {
        kg::kv_commit(st, s.dtype == KOALA_BF16, c->kv.target_k, c->kv.target_v, c->kv.ctx_len, accept_len,
                      accept_path, c->D, s.n_layers, c->max_batch, batch, s.n_heads, c->kv.capacity, s.head_dim);
        kg::advance_ctx(st, c->kv.ctx_len, accept_len, batch);
    }
    KOALA_CHECK_LAUNCH(c);
    return KOALA_OK;
}

koala_status koala_accept_sample(koala_ctx *c, void *hip_stream, int batch, const int32_t *tree_tokens,
                                 const float *target_logits, const float *draft_logits, const float *u_accept,
                                 const float *u_resample, float temperature, int32_t *accept_len,
                                 int32_t *accept_path, int32_t *next_token, int commit) {
    return accept_sample_impl(c, hip_stream, batch, tree_tokens, target_logits, draft_logits, u_accept, u_resample,
                              temperature, accept_len, accept_path, next_token, commit, false);
}

koala_status koala_accept_sample_static(koala_ctx *c, void *hip_stream, int batch, const int32_t *tree_tokens,
                                        const float *target_logits, const float *draft_logits,
                                        const float *u_accept, const float *u_resample, float temperature,
                                        int32_t *accept_len, int32_t *accept_path, int32_t *next_token,
                                        int commit) {
    return accept_sample_impl(c, hip_stream, batch, tree_tokens, target_logits, draft_logits, u_accept, u_resample,
                              temperature, accept_len, accept_path, next_token, commit, true);
}

koala_status koala_accept_prefix(koala_ctx *c, void *hip_stream, int batch, const int32_t *tree_tokens,
                                 const int32_t *greedy, int32_t *accept_len, int32_t *accept_path,
                                 int32_t *next_token, int commit) {
    koala_status st0 = check_call(c, batch);
    if (st0 != KOALA_OK) return st0;
    if (!tree_tokens || !greedy || !accept_len || !accept_path || !next_token)
        return fail(c, KOALA_E_NULL, "all accept_prefix pointers are required");
    hipStream_t st = (hipStream_t)hip_stream;
    const koala_shape &s = c->shape;
    kg::accept_scan(st, c->tt, c->T, c->D, tree_tokens, greedy, accept_len, accept_path, next_token, batch);
    if (commit) {
        kg::kv_commit(st, s.dtype == KOALA_BF16, c->kv.target_k, c->kv.target_v, c->kv.ctx_len, accept_len,
                      accept_path, c->D, s.n_layers, c->max_batch, batch, s.n_heads, c->kv.capacity, s.head_dim);
        kg::advance_ctx(st, c->kv.ctx_len, accept_len, batch);
    }
    KOALA_CHECK_LAUNCH(c);
    return KOALA_OK;
}

// uniforms == nullptr: greedy loop.  Otherwise iteration i draws with uniforms[i][0..2][n_nodes]
// (children, acceptance, replacement) at the given temperature; at most max_iters iterations.
static koala_status generate_impl(koala_ctx *c, void *hip_stream, const float *feat_in, const int32_t *tok_in, int m,
                                  int ctx_len0, int max_new, int use_draft, const float *uniforms, int max_iters,
                                  float temperature, int32_t *out_tokens, koala_gen_stats *stats) {
    koala_status st0 = check_call(c, 1);
    if (st0 != KOALA_OK) return st0;
    const bool sampling = uniforms != nullptr;
    const int Tp = (c->T + 3) & ~3;   // row stride of the uniforms: rows stay 16-byte aligned
    if (sampling) {
        if (!use_draft) return fail(c, KOALA_E_UNSUPPORTED, "non-greedy generation needs a draft head");
        if (!(temperature > 0.f)) return fail(c, KOALA_E_SHAPE, "temperature must be positive");
        if (max_iters < 1) return fail(c, KOALA_E_SHAPE, "max_iters must be positive");
        if (!aligned16(uniforms)) return fail(c, KOALA_E_ALIGN, "uniforms must be 16-byte aligned");
    }
    if (!tok_in || !out_tokens || !stats || (use_draft && !feat_in))
        return fail(c, KOALA_E_NULL, "generate: tok_in, out_tokens and stats are required (feat_in too when drafting)");
    const koala_shape &s = c->shape;
    const bool eagle = c->draft.kind == KOALA_DRAFT_EAGLE;
    if (m < 1 || m > c->draft.max_m) return fail(c, KOALA_E_SHAPE, "generate: m must be in 1..max_m");
    if (max_new < 1) return fail(c, KOALA_E_SHAPE, "generate: max_new must be positive");
    if (!use_draft && c->T != 1)
        return fail(c, KOALA_E_SHAPE, "generate: plain decoding (use_draft = 0) needs a single-node tree");
    if (use_draft && eagle && c->draft.max_m < c->D + 1)
        return fail(c, KOALA_E_SHAPE, "generate: the draft head needs max_m >= depth + 1 catch-up rows");
    // every iteration needs rows C .. C + n_nodes - 1 of the caches; C grows by at most depth + 1 per iteration
    if (ctx_len0 < m || (long long)ctx_len0 + max_new + c->D + c->T > c->kv.capacity)
        return fail(c, KOALA_E_SHAPE, "generate: ctx_len0 + max_new + depth + n_nodes exceeds the cache capacity");
    hipStream_t st = (hipStream_t)hip_stream;
    memset(stats, 0, sizeof(*stats));
    {
        int32_t c_dev = -1;
        if (hipMemcpyAsync(&c_dev, c->kv.ctx_len, sizeof(c_dev), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            return fail(c, KOALA_E_DEVICE, "generate: reading ctx_len[0] failed");
        if (c_dev != ctx_len0) return fail(c, KOALA_E_SHAPE, "generate: ctx_len0 differs from ctx_len[0] on the device");
    }
    if (hipMemcpyAsync(c->gen_tok_in, tok_in, (size_t)m * sizeof(int32_t), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(c, KOALA_E_DEVICE, "generate: copy of tok_in failed");
    if (use_draft && hipMemcpyAsync(c->gen_feat_in, feat_in, (size_t)m * s.hidden * sizeof(float),
                                    hipMemcpyDeviceToDevice, st) != hipSuccess)
        return fail(c, KOALA_E_DEVICE, "generate: copy of feat_in failed");
    int n_done = 0, cur_m = m;
    while (n_done < max_new) {
        koala_status r;
        const float *u = nullptr;
        if (sampling) {
            if (stats->iterations >= max_iters)
                return fail(c, KOALA_E_CAPACITY, "generate: max_iters iterations were not enough for max_new tokens");
            u = uniforms + (size_t)stats->iterations * 3 * Tp;
            r = koala_draft_expand_sample(c, st, 1, c->gen_feat_in, c->gen_tok_in, cur_m, u, temperature, c->gen_tree,
                                          c->gen_dlogits);
            if (r != KOALA_OK) return r;
        } else if (use_draft) {
            r = koala_draft_expand(c, st, 1, c->gen_feat_in, c->gen_tok_in, cur_m, c->gen_tree, nullptr);
            if (r != KOALA_OK) return r;
        } else {
            kg::set_root(st, c->gen_tok_in, cur_m, c->gen_tree, nullptr, 1, c->T);
        }
        r = koala_tree_verify(c, st, 1, c->gen_tree, c->gen_feat, sampling ? c->gen_tlogits : nullptr, c->gen_greedy);
        if (r != KOALA_OK) return r;
        r = sampling ? koala_accept_sample(c, st, 1, c->gen_tree, c->gen_tlogits, c->gen_dlogits, u + Tp,
                                           u + 2 * Tp, temperature, c->gen_acc, c->gen_path, c->gen_next, 1)
                     : koala_accept_prefix(c, st, 1, c->gen_tree, c->gen_greedy, c->gen_acc, c->gen_path, c->gen_next,
                                           1);
        if (r != KOALA_OK) return r;
        kg::gen_next(st, c->gen_feat, c->gen_tree, c->gen_acc, c->gen_path, c->gen_next, c->T, c->D, s.hidden,
                     c->gen_feat_in, c->gen_tok_in, out_tokens, n_done, max_new);
        KOALA_CHECK_LAUNCH(c);
        int32_t a = -1;
        if (hipMemcpyAsync(&a, c->gen_acc, sizeof(a), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            return fail(c, KOALA_E_DEVICE, "generate: reading the accepted length failed");
        if (a < 0 || a > c->D) return fail(c, KOALA_E_DEVICE, "generate: accepted length out of range");
        stats->accept_hist[a] += 1;
        stats->iterations += 1;
        n_done += a + 1;
        cur_m = eagle && use_draft ? a + 1 : 1;
        if (!(eagle && use_draft) && a > 0) {
            // only the newest row is needed: move row a of the next inputs to row 0
            if (hipMemcpyAsync(c->gen_tok_in, c->gen_tok_in + a, sizeof(int32_t), hipMemcpyDeviceToDevice, st) != hipSuccess ||
                hipMemcpyAsync(c->gen_feat_in, c->gen_feat_in + (size_t)a * s.hidden, (size_t)s.hidden * sizeof(float),
                               hipMemcpyDeviceToDevice, st) != hipSuccess)
                return fail(c, KOALA_E_DEVICE, "generate: moving the newest row failed");
        }
    }
    stats->tokens = n_done;
    return KOALA_OK;
}

koala_status koala_generate(koala_ctx *c, void *hip_stream, const float *feat_in, const int32_t *tok_in, int m,
                            int ctx_len0, int max_new, int use_draft, int32_t *out_tokens, koala_gen_stats *stats) {
    return generate_impl(c, hip_stream, feat_in, tok_in, m, ctx_len0, max_new, use_draft, nullptr, 0, 1.f, out_tokens,
                         stats);
}

koala_status koala_generate_sample(koala_ctx *c, void *hip_stream, const float *feat_in, const int32_t *tok_in,
                                   int m, int ctx_len0, int max_new, const float *uniforms, int max_iters,
                                   float temperature, int32_t *out_tokens, koala_gen_stats *stats) {
    if (c && !uniforms) return fail(c, KOALA_E_NULL, "uniforms are required");
    return generate_impl(c, hip_stream, feat_in, tok_in, m, ctx_len0, max_new, 1, uniforms, max_iters, temperature,
                         out_tokens, stats);
}

koala_status koala_weights_to_half(void *hip_stream, void *packed, size_t n_elements) {
    if (!packed) return KOALA_E_NULL;
    if (n_elements % 8) return KOALA_E_SHAPE;
    if ((uintptr_t)packed & 15) return KOALA_E_ALIGN;
    kb::weights_to_f16((hipStream_t)hip_stream, packed, n_elements);
    return hipGetLastError() == hipSuccess ? KOALA_OK : KOALA_E_DEVICE;
}

koala_status koala_measure_stream_read(void *hip_stream, const void *buffer, size_t bytes, void *sink, int repeats,
                                       double *gb_per_s) {
    if (!buffer || !gb_per_s || !sink) return KOALA_E_NULL;
    if (bytes < 16 || repeats < 1) return KOALA_E_SHAPE;
    if (((uintptr_t)buffer & 15) || ((uintptr_t)sink & 15)) return KOALA_E_ALIGN;
    hipStream_t st = (hipStream_t)hip_stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    koala_status rc = KOALA_E_DEVICE;
    if (hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess) {
        kg::stream_read(st, buffer, bytes, (unsigned *)sink);   // warm-up
        bool ok = hipEventRecord(e0, st) == hipSuccess;
        for (int r = 0; r < repeats; ++r) kg::stream_read(st, buffer, bytes, (unsigned *)sink);
        float ms = 0.f;
        ok = ok && hipEventRecord(e1, st) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
             hipEventElapsedTime(&ms, e0, e1) == hipSuccess && hipGetLastError() == hipSuccess;
        if (ok && ms > 0.f) {
            *gb_per_s = (double)(bytes / 16 * 16) * repeats / (ms * 1e-3) / 1e9;
            rc = KOALA_OK;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    return rc;
}

koala_status koala_profile_begin(koala_ctx *c, int max_launches) {
    if (!c) return KOALA_E_NULL;
    c->err.clear();
    if (max_launches < 1 || max_launches > (1 << 16)) return fail(c, KOALA_E_SHAPE, "max_launches out of range");
    while (c->prof_ev.size() < (size_t)2 * max_launches) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return fail(c, KOALA_E_DEVICE, "hipEventCreate failed");
        c->prof_ev.push_back(e);
    }
    c->prof_used = 0;
    c->prof_bytes = 0.0;
    c->prof_on = true;
    return KOALA_OK;
}

koala_status koala_profile_end(koala_ctx *c, double *gemm_ms, int *gemm_launches, double *gemm_bytes) {
    if (!c) return KOALA_E_NULL;
    c->err.clear();
    c->prof_on = false;
    double total = 0.0;
    for (int i = 0; i + 1 < c->prof_used; i += 2) {
        float ms = 0.f;
        if (hipEventSynchronize(c->prof_ev[i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, c->prof_ev[i], c->prof_ev[i + 1]) != hipSuccess)
            return fail(c, KOALA_E_DEVICE, "reading profile events failed");
        total += ms;
    }
    if (gemm_ms) *gemm_ms = total;
    if (gemm_launches) *gemm_launches = c->prof_used / 2;
    if (gemm_bytes) *gemm_bytes = c->prof_bytes;
    c->prof_used = 0;
    return KOALA_OK;
}

const char *koala_last_error(const koala_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

void koala_destroy(koala_ctx *ctx) {
    if (!ctx) return;
    for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
    delete ctx;
}

}  // extern "C"
