/*
 * koala.h - C ABI of the draft-then-verify hot path of multi-layer-draft-head
 * speculative decoding on one AMD MI355X (gfx950).
 *
 * One iteration (paper section 2.2): a K-layer draft head proposes candidate
 * tokens arranged in a static tree (Eq. 2; EAGLE-style or Medusa-style head,
 * section 3.1), the target model scores all of them in one pass (Eq. 3), and
 * the longest root path whose tokens equal the target's greedy choices is kept
 * together with the target's own next token (sections 2.2 and 4.1).
 *
 * General rules
 *  - "device" pointers are HIP device memory owned by the caller; "host"
 *    pointers are ordinary host memory.  The library allocates no device
 *    memory: all scratch lives in the caller's workspace (koala_bind), except
 *    for the fixed array of koala_accept_sample_static, which is part of the
 *    loaded library itself.
 *  - Tensors are dense, row-major, 16-byte aligned.  Weights and KV caches are
 *    stored in the model dtype (fp32 or bfloat16); features, logits and scores
 *    are always fp32; token ids, node ids and lengths are int32.
 *  - Linear layers are [out_features, in_features] and have no bias.
 *  - The iteration calls (draft_expand, tree_verify, accept_prefix and their
 *    non-greedy counterparts) only enqueue work on the given hipStream_t
 *    (passed as void*); they never synchronise and never read results back, so
 *    they can be captured into a HIP graph.  koala_generate and the measurement
 *    aids are the exceptions and say so.  Calls on one context must be issued
 *    on one stream, or otherwise ordered by the caller; a context is not safe
 *    for concurrent use from several host threads.
 *  - Arguments are validated on the host before anything is launched; a call
 *    that returns an error has had no effect on device memory (koala_generate:
 *    none from the failing iteration on; earlier iterations stay committed).  Errors are
 *    returned as negative koala_status values; koala_last_error() gives text.
 *  - Limits: at most 64 tree nodes per sequence, at most 64 catch-up rows (m),
 *    head_dim 64 or 128, hidden = n_heads * head_dim; for bfloat16 hidden and
 *    ffn must be multiples of 128 and vocab at most 65536.
 *
 * Matrix storage.  For KOALA_FP32 every matrix [N, K] is plain row-major.  For
 * KOALA_BF16 every Linear weight (wqkv, wo, wgu, wdown, lm_head, fc, Medusa
 * blocks) is stored "fragment-major", the order in which a gfx950 wave feeds a
 * 16x16x32 MFMA, so that the weight stream is read from HBM as contiguous
 * 1 KiB pieces.  With Npad = N rounded up to a multiple of 64 (extra rows zero)
 * and K a multiple of 64, element (n, k) lives at 16-bit index
 *     (((((n/64) * (K/64) + k/64) * 4 + (n%64)/16) * 2 + (k%64)/32) * 64
 *        + (n%16) + 16*((k%32)/8)) * 8 + k%8,
 * i.e. tiles of 64 rows x 64 k, each tile being 8 fragments of 64 lanes x 8
 * values.  The matrix pipe multiplies in fp16 (with fp32 accumulation): a matrix
 * laid out this way in bfloat16 is handed to koala_weights_to_half once, which
 * rewrites it in place as fp16 (the same values: a bfloat16 number has eight
 * significant bits, fp16 holds eleven), and it is that form koala_bind takes.
 * The embedding table, the RMSNorm gains and the KV caches stay bfloat16,
 * row-major / linear.
 *
 * Arithmetic of the KOALA_BF16 path.  Every projection multiplies fp16 by fp16
 * and accumulates in fp32: its input (the normalised hidden state times the
 * norm's gain, the attention output, SiLU(gate) * up) is rounded to fp16 where
 * the producing kernel writes it, and a value beyond +-65504 saturates there.
 * Attention multiplies the bfloat16 cache rows with queries and probabilities
 * carried as bfloat16 hi + lo pairs; softmax, normalisation, residual stream,
 * logits and features are fp32.
 */
#ifndef KOALA_H
#define KOALA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct koala_ctx koala_ctx; /* opaque, host-side */

typedef enum {
    KOALA_OK = 0,
    KOALA_E_NULL = -1,        /* a required pointer is NULL */
    KOALA_E_SHAPE = -2,       /* inconsistent sizes, malformed tree, batch/m out of range */
    KOALA_E_ALIGN = -3,       /* a device pointer is not 16-byte aligned */
    KOALA_E_CAPACITY = -4,    /* KV capacity cannot hold context + tree rows */
    KOALA_E_UNSUPPORTED = -5, /* dtype / head_dim / draft kind not implemented */
    KOALA_E_WORKSPACE = -6,   /* workspace missing or too small, or context not bound */
    KOALA_E_DEVICE = -7       /* a HIP call or kernel launch failed */
} koala_status;

enum { KOALA_FP32 = 0, KOALA_BF16 = 1 };
enum { KOALA_DRAFT_EAGLE = 0, KOALA_DRAFT_MEDUSA = 1 };
enum { KOALA_MAX_NODES = 64, KOALA_MAX_M = 64 };

/* Llama-style decoder stack of the target model (section 4.1). */
typedef struct {
    int hidden, n_heads, head_dim, ffn, vocab, n_layers;
    float rms_eps, rope_base;
    int dtype; /* KOALA_FP32 or KOALA_BF16: storage type of weights and KV caches */
} koala_shape;

/* Draft head (section 3.1).  EAGLE-style: Linear over [embedding ; feature]
 * followed by K decoder layers of the target's shape, sharing the target's
 * embedding and LM head.  Medusa-style: medusa_heads heads, head j being K
 * residual blocks x <- x + SiLU(W x) followed by the shared LM head; head j
 * fills tree depth j+1, so medusa_heads must be >= tree depth. */
typedef struct {
    int kind;         /* KOALA_DRAFT_EAGLE or KOALA_DRAFT_MEDUSA */
    int K;            /* layers per head, >= 1 */
    int medusa_heads; /* Medusa only */
    int max_m;        /* largest m passed to koala_draft_expand (1..KOALA_MAX_M) */
} koala_draft_shape;

/* Static candidate tree; host arrays, copied by koala_create.  Node 0 is the
 * root (the newest committed token); parent[0] = -1 and parent[i] < i; nodes
 * are ordered by depth.  rank[i] says which of its parent's top-k tokens node i
 * receives (0 = most likely); siblings have distinct ranks below
 * topk_per_depth[depth(i) - 1]. */
typedef struct {
    int n_nodes, depth;
    const int32_t *parent;         /* host int32[n_nodes] */
    const int32_t *rank;           /* host int32[n_nodes] */
    const int32_t *topk_per_depth; /* host int32[depth] */
} koala_tree;

/* Device weight pointers, borrowed until koala_destroy or the next koala_bind.
 *   embed, lm_head  [vocab, hidden];  final_norm [hidden]
 *   layer_w: host array of 6 * n_layers device pointers, per layer
 *       in_norm [hidden], wqkv [3*hidden, hidden] (rows: all of W_q, then W_k, then W_v; for KOALA_BF16
 *           the rows of W_q and W_k are reordered inside every head so that the two members of a rotary
 *           pair are neighbours: row 2i of a head is dimension i, row 2i+1 is dimension i + head_dim/2),
 *       wo [hidden, hidden], post_norm [hidden],
 *       wgu [2*ffn, hidden] with rows interleaved (row 2f = gate_f, row 2f+1 = up_f),
 *       wdown [hidden, ffn]
 *   EAGLE: fc [hidden, 2*hidden] acting on [embedding ; feature];
 *          draft_w: host array of 6 * K pointers, same per-layer order as layer_w
 *   Medusa: fc = NULL; draft_w: host array of medusa_heads * K pointers,
 *          draft_w[j*K + k] = W_{j,k} [hidden, hidden] */
typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void *const *layer_w;
    const void *fc;
    const void *const *draft_w;
} koala_weights;

/* KV caches, device, model dtype, layout [layer][batch][n_heads][capacity][head_dim]
 * (target: n_layers layers; EAGLE draft: K layers; Medusa: draft_k = draft_v = NULL).
 * Keys are stored already rotated.  ctx_len: device int32[max_batch]; ctx_len[b]
 * = number of committed rows C_b of sequence b in the target cache.  Rows
 * C_b .. C_b + n_nodes - 1 are scratch for the tree, so capacity must always be
 * >= C_b + n_nodes (the caller's responsibility: C_b lives on the device).  The
 * caches must hold finite numbers everywhere (e.g. be zero-filled once after
 * allocation): scratch rows are read, with weight zero, before they are written. */
typedef struct {
    void *target_k, *target_v, *draft_k, *draft_v;
    int capacity;
    int32_t *ctx_len;
} koala_kv;

/* Create a context for a model shape, draft head and tree.  Host only. */
koala_status koala_create(const koala_shape *shape, const koala_draft_shape *draft,
                          const koala_tree *tree, int max_batch, koala_ctx **out);

/* Bytes of device workspace koala_bind needs for this context. */
koala_status koala_workspace_bytes(const koala_ctx *ctx, size_t *out);

/* Attach weights, KV caches and a device workspace (>= koala_workspace_bytes,
 * 256-byte aligned).  Copies the tree tables into the workspace with a
 * synchronous host-to-device copy.  The workspace contents belong to the
 * library until koala_destroy. */
koala_status koala_bind(koala_ctx *ctx, const koala_weights *w, const koala_kv *kv,
                        void *workspace, size_t workspace_bytes);

/* Draft step (Eq. 2).  For each sequence b < batch:
 *   feat_in  device fp32 [batch, m, hidden]: target features (hidden state after
 *            the final RMSNorm) of the m newest committed positions C_b-m .. C_b-1;
 *   tok_in   device int32 [batch, m]: the token following each of them;
 *            tok_in[b, m-1] is the newest committed token = tree root.
 * EAGLE: the draft cache must hold rows 0 .. C_b-m-1; rows C_b-m .. C_b-1 are
 * computed first (row i pairs feature i with token i+1 at position i), then the
 * tree is expanded depth by depth: every node that has children is run through
 * the head at position C_b-1+depth, attending to the draft context and its own
 * ancestors, and its top-k tokens (descending logit, ties to the lower id) go
 * to its children by rank.  Draft-cache rows >= C_b are scratch afterwards.
 * Medusa: only feat_in[b, m-1] is used.
 *   tree_tokens device int32 [batch, n_nodes] (out): token of every node, root included;
 *   tree_scores device fp32 [batch, n_nodes] (out, may be NULL): draft logit of
 *            each node's token under its parent (root: 0). */
koala_status koala_draft_expand(koala_ctx *ctx, void *hip_stream, int batch,
                                const float *feat_in, const int32_t *tok_in, int m,
                                int32_t *tree_tokens, float *tree_scores);

/* Verification (Eq. 3).  Runs the target on all n_nodes rows of each sequence:
 * node i is at position C_b + depth(i), its key/value are written to cache slot
 * C_b + i of every layer, and it attends to the C_b context rows plus itself
 * and its ancestors.
 *   tree_tokens device int32 [batch, n_nodes];
 *   feat_out    device fp32 [batch, n_nodes, hidden] (out): features after the final RMSNorm;
 *   logits_out  device fp32 [batch, n_nodes, vocab] (out, may be NULL);
 *   greedy_out  device int32 [batch, n_nodes] (out): argmax of each row's logits,
 *               lowest id among equal maxima. */
koala_status koala_tree_verify(koala_ctx *ctx, void *hip_stream, int batch,
                               const int32_t *tree_tokens, float *feat_out, float *logits_out,
                               int32_t *greedy_out);

/* Greedy acceptance (sections 2.2, 4.1).  Starting at the root, repeatedly step
 * to the lowest-numbered child whose token equals greedy[current]; stop when
 * there is none.
 *   accept_len  device int32 [batch] (out): number of accepted drafted tokens a, 0..depth;
 *   accept_path device int32 [batch, depth+1] (out): node ids root..last accepted, then -1;
 *   next_token  device int32 [batch] (out): greedy[last accepted node];
 *   commit != 0: additionally, in every target layer, copy the key/value rows of
 *               the path nodes to slots C_b .. C_b+a and set ctx_len[b] += a+1. */
koala_status koala_accept_prefix(koala_ctx *ctx, void *hip_stream, int batch,
                                 const int32_t *tree_tokens, const int32_t *greedy,
                                 int32_t *accept_len, int32_t *accept_path, int32_t *next_token,
                                 int commit);

/* Non-greedy drafting (section 2.2: the drafted tokens are drawn from the draft distributions;
 * section 4.4 evaluates temperature 1).  As koala_draft_expand, but the
 * children of a node are draws without replacement from softmax(draft logits at the node /
 * temperature): the child of lowest rank is drawn first, each later one from what is left after
 * removing the earlier draws, by inverse CDF over ascending token id (first id at which the
 * running sum exceeds u * total).
 *   u_draw       device fp32 [batch, n_nodes]: uniform in [0,1) used for the draw of each node
 *                (entry 0, the root, is not used);
 *   draft_logits device fp32 [batch, n_nodes, vocab] (out): row i = draft logits at node i, written
 *                for the nodes that have children; koala_accept_sample reads them.
 * Medusa-style heads: the head of depth j gives one distribution for all nodes of that depth;
 * every parent draws its own children from it (with its children's uniforms), and row i of
 * draft_logits is the logits of the head that drafts node i's children. */
koala_status koala_draft_expand_sample(koala_ctx *ctx, void *hip_stream, int batch,
                                       const float *feat_in, const int32_t *tok_in, int m,
                                       const float *u_draw, float temperature,
                                       int32_t *tree_tokens, float *draft_logits);

/* Stochastic acceptance (section 2.2), per sequence: at the current node, with q = softmax(target
 * logits / temperature) and d = softmax(draft logits / temperature), try the children in draw
 * order: child with token x is accepted if u_accept[child] < min(1, q(x)/d(x)) and becomes the
 * current node; after a rejection q <- norm(max(0, q - d)) (unchanged if that is all zero), x is
 * removed from d and d renormalised.  Where no child is accepted, or the node has none,
 * next_token is drawn from q by inverse CDF with u_resample[node].  On a chain template this is
 * the rule of section 2.2 as printed; trying several children in turn is this build's reading for
 * trees.  With the children drawn by koala_draft_expand_sample the emitted tokens are distributed
 * as the target's own samples.
 *   target_logits device fp32 [batch, n_nodes, vocab]: logits_out of koala_tree_verify;
 *   draft_logits  device fp32 [batch, n_nodes, vocab]: from koala_draft_expand_sample;
 *   u_accept, u_resample device fp32 [batch, n_nodes]: uniforms in [0,1);
 *   outputs and commit as in koala_accept_prefix. */
koala_status koala_accept_sample(koala_ctx *ctx, void *hip_stream, int batch,
                                 const int32_t *tree_tokens, const float *target_logits,
                                 const float *draft_logits, const float *u_accept,
                                 const float *u_resample, float temperature, int32_t *accept_len,
                                 int32_t *accept_path, int32_t *next_token, int commit);

/* koala_accept_sample for callers that cannot allocate device memory or size a workspace for it: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Identical to
 * koala_accept_sample (same kernels, same results bit for bit) except that the two vocabulary-sized
 * distributions per sequence that the walk keeps are held in a fixed array inside the library
 * (2 MiB of device memory per GPU, present from the moment the library is loaded until the process
 * ends) instead of the workspace.  The call allocates nothing.
 *   Limit: batch * vocab <= 262144, else KOALA_E_CAPACITY (nothing is launched).
 *   The array is shared by every context and every call on the same GPU: two calls that overlap on
 *   one GPU (different streams or threads) race; calls on one stream are ordered.  Nothing in the
 *   array has to be cleared between calls (every element a call reads, it has written before). */
koala_status koala_accept_sample_static(koala_ctx *ctx, void *hip_stream, int batch,
                                        const int32_t *tree_tokens, const float *target_logits,
                                        const float *draft_logits, const float *u_accept,
                                        const float *u_resample, float temperature,
                                        int32_t *accept_len, int32_t *accept_path,
                                        int32_t *next_token, int commit);

/* Statistics of a generation run.  accept_hist[a] counts the iterations that accepted exactly a
 * drafted tokens; from it follow the average number of tokens per iteration (section 4.1:
 * sum_a (a+1) accept_hist[a] / iterations) and, for a chain template, the n-alpha acceptance rates
 * (section 4.1: alpha_n = #{a >= n} / #{a >= n-1}). */
typedef struct {
    int32_t iterations;       /* draft-verify iterations run */
    int32_t tokens;           /* tokens produced by them, >= max_new */
    int32_t accept_hist[64];
} koala_gen_stats;

/* Generation loop on sequence 0 (section 2.2 repeated; metrics of section 4.1): repeat
 * draft_expand -> tree_verify -> accept_prefix(commit), feeding the features and tokens of the
 * accepted path back as the next call's catch-up rows, until max_new tokens have been produced.
 * Preconditions are those of koala_draft_expand for the first call: the target cache holds
 * rows 0 .. ctx_len0-1, an EAGLE draft cache rows 0 .. ctx_len0-m-1, and
 *   feat_in device fp32 [m, hidden], tok_in device int32 [m] as in koala_draft_expand
 *           (tok_in[m-1] is the root of the first tree);
 *   ctx_len0 the value of ctx_len[0] on the device (checked), with
 *           ctx_len0 + max_new + depth + n_nodes <= capacity;
 *   use_draft = 0: plain autoregressive decoding with the target only (the baseline of the
 *           speed-up ratio in section 4.1); the context must have a single-node tree, feat_in is
 *           ignored and every iteration yields one token;
 *   out_tokens device int32 [max_new] (out): the tokens produced, in order (tok_in[m-1] itself is
 *           not repeated);
 *   stats   host (out).
 * An EAGLE context needs max_m >= depth + 1.  The accepted length of every iteration is read
 * back (one 4-byte copy and a stream synchronisation per iteration), so the call returns with
 * the stream idle.  Uses buffers inside the workspace; batch > 1 is not supported here. */
koala_status koala_generate(koala_ctx *ctx, void *hip_stream, const float *feat_in,
                            const int32_t *tok_in, int m, int ctx_len0, int max_new, int use_draft,
                            int32_t *out_tokens, koala_gen_stats *stats);

/* Non-greedy generation loop (sections 2.2 and 4.4): as koala_generate with a draft head of either
 * kind, but every iteration is koala_draft_expand_sample -> koala_tree_verify -> koala_accept_sample
 * (commit) at the given temperature.
 *   uniforms device fp32 [max_iters, 3, n_nodes_padded], n_nodes_padded = n_nodes rounded up to a
 *            multiple of 4: iteration i uses row [i,0] as u_draw, [i,1] as u_accept, [i,2] as
 *            u_resample (entries >= n_nodes unused);
 *   max_iters: KOALA_E_CAPACITY is returned (iterations so far stay committed) if that many
 *            iterations did not produce max_new tokens; max_iters >= max_new always suffices.
 * tok_in[m-1], the root of the first tree, is the caller's choice (e.g. its own draw from the
 * prefill's last distribution).  Other arguments, outputs and statistics as in koala_generate. */
koala_status koala_generate_sample(koala_ctx *ctx, void *hip_stream, const float *feat_in,
                                   const int32_t *tok_in, int m, int ctx_len0, int max_new,
                                   const float *uniforms, int max_iters, float temperature,
                                   int32_t *out_tokens, koala_gen_stats *stats);

/* Linear weights of the bfloat16 path, once, before koala_bind (see "Matrix storage"): `packed` is a
 * fragment-major matrix of n_elements bfloat16 values in device memory (16-byte aligned, n_elements a
 * multiple of 8) and is rewritten in place as fp16 by a kernel enqueued on the stream.  Exact for
 * magnitudes from 2^-24 to 65504; smaller values round to the nearest multiple of 2^-24, larger ones
 * become infinite.  Calling it twice on the same matrix destroys it.  No koala_ctx is needed. */
koala_status koala_weights_to_half(void *hip_stream, void *packed, size_t n_elements);

/* Measurement aid (not part of the method): the rate at which this device streams `bytes` of
 * `buffer` (device memory, 16-byte aligned) through a plain read kernel with the same load
 * instructions the weight-streaming GEMM uses, averaged over `repeats` back-to-back launches after
 * one warm-up; the attainable counterpart of the nominal HBM peak.  `sink` is 256 bytes of device
 * memory of the caller's (16-byte aligned) that the kernel may write to.  Synchronises on its own
 * events.  Host only. */
koala_status koala_measure_stream_read(void *hip_stream, const void *buffer, size_t bytes,
                                       void *sink, int repeats, double *gb_per_s);

/* Measurement aid for benchmarks (not part of the method).  Between koala_profile_begin and
 * koala_profile_end every weight-streaming GEMM launch of the bfloat16 path carries a pair
 * of HIP events bound to its own dispatch on the call's stream, which take the kernel's begin and
 * end times (at most max_launches pairs; further launches are not timed).  koala_profile_end synchronises on the recorded events and returns the summed kernel
 * time in milliseconds, the number of timed launches and the weight bytes those launches
 * streamed (their algorithmic HBM traffic).  Host only; any out pointer may be NULL. */
koala_status koala_profile_begin(koala_ctx *ctx, int max_launches);
koala_status koala_profile_end(koala_ctx *ctx, double *gemm_ms, int *gemm_launches, double *gemm_bytes);

/* ---------------------------------------------------------------------------------------------
 * Adversarial training step of a draft head (section 3.2, Algorithm 1).  These calls need no koala_ctx:
 * every tensor is a dense row-major fp32 device array of the caller's, the calls only enqueue kernels on
 * the given stream, and parameters are updated in place by plain gradient descent.
 *
 * The discriminator D (section 3.2: a linear layer followed by fully connected layers, as many as the
 * draft head has layers) scores a row of token logits together with the target model's last hidden
 * state h of that position: z = W_lin h (hidden -> vocab), u = z + logits, then n_fc fully connected
 * layers with biases, ReLU between them, the last of width 1, and a sigmoid: D = sigmoid(s).  How the
 * mapped hidden state and the logits are joined, the widths, the biases and the activation are this
 * build's readings (the paper names the layers only); expectations are means over the n_rows positions.
 * --------------------------------------------------------------------------------------------- */
typedef struct {
    int hidden, vocab;
    int fc_hidden; /* width of the inner fully connected layers (unused when n_fc = 1) */
    int n_fc;      /* fully connected layers, 1..3: vocab -> fc_hidden -> .. -> 1 */
} koala_disc_shape;

/* w_lin [vocab, hidden]; w_fc[k] [out_k, in_k] and b_fc[k] [out_k] with in_0 = vocab, inner widths
 * fc_hidden, out of the last layer = 1; entries k >= n_fc are ignored. */
typedef struct {
    float *w_lin;
    float *w_fc[3];
    float *b_fc[3];
} koala_disc_params;

/* Bytes of device workspace the two discriminator calls need for n_rows positions. */
koala_status koala_train_workspace_bytes(const koala_disc_shape *shape, int n_rows, size_t *out);

/* Discriminator step (Algorithm 1, Eq. 6): L_D = -mean log(1 - D(d)) - mean log D(q) over the n_rows
 * positions, its gradient with respect to every discriminator parameter, and params <- params - lr * grad
 * (lr = 0: loss only).  h [n_rows, hidden], q_logits / d_logits [n_rows, vocab] (the target's and the draft
 * head's logits of the same positions); loss_out device fp32 [1]: L_D before the update. */
koala_status koala_train_disc_step(const koala_disc_shape *shape, const koala_disc_params *params,
                                   void *hip_stream, int n_rows, const float *h, const float *q_logits,
                                   const float *d_logits, float lr, void *workspace,
                                   size_t workspace_bytes, float *loss_out);

/* Draft-head side (Algorithm 1, Eq. 5) at the logits: L_G = -lambda * mean log D(d) + L_Distill(d, q) with
 * L_Distill the cross-entropy of softmax(d) against softmax(q) (mean over positions).
 *   loss_out device fp32 [2] (out): the adversarial term and the distillation term;
 *   grad_d   device fp32 [n_rows, vocab] (out): dL_G / dd, what the draft head's backward pass starts from.
 * The discriminator's parameters are read only. */
koala_status koala_train_gen_grad(const koala_disc_shape *shape, const koala_disc_params *params,
                                  void *hip_stream, int n_rows, const float *h, const float *q_logits,
                                  const float *d_logits, float lambda, void *workspace,
                                  size_t workspace_bytes, float *loss_out, float *grad_d);

/* A Medusa-style head in training (section 3.1: K residual blocks x <- x + SiLU(W_k x) followed by the
 * target's LM head, which stays fixed): blocks_w host array of K device pointers to W_k [hidden, hidden],
 * w_lm [vocab, hidden], h [n_rows, hidden].
 *   _forward: d_logits [n_rows, vocab] (out) = the head's logits;
 *   _step:    given grad_d = dL_G / dd (koala_train_gen_grad), the head's backward pass and
 *             W_k <- W_k - lr * dL_G/dW_k for every block (the draft-head update of Algorithm 1).
 * An EAGLE-style head's backward pass (decoder layers with attention) is not provided.  K <= 8. */
koala_status koala_train_medusa_workspace_bytes(int n_rows, int hidden, int K, size_t *out);
koala_status koala_train_medusa_head_forward(void *hip_stream, int n_rows, int hidden, int vocab, int K,
                                             float *const *blocks_w, const float *w_lm, const float *h,
                                             void *workspace, size_t workspace_bytes, float *d_logits);
koala_status koala_train_medusa_head_step(void *hip_stream, int n_rows, int hidden, int vocab, int K,
                                          float *const *blocks_w, const float *w_lm, const float *h,
                                          const float *grad_d, float lr, void *workspace,
                                          size_t workspace_bytes);

/* Text of the last error on this context ("" if none); valid until the next call. */
const char *koala_last_error(const koala_ctx *ctx);

void koala_destroy(koala_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* KOALA_H */
