// Straightforward fp32-arithmetic kernels for every step of the draft-then-verify
// iteration.  They serve the fp32 model dtype and all the small bookkeeping steps;
// the bf16 weight-streaming GEMMs and attention have dedicated kernels elsewhere.
#include "koala_internal.h"

namespace {

__device__ __forceinline__ float ldf(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const bf16_t *p, size_t i) {
    return __uint_as_float(((uint32_t)p[i]) << 16);
}
__device__ __forceinline__ void stf(float *p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void stf(bf16_t *p, size_t i, float v) {  // round to nearest even
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    p[i] = (bf16_t)(u >> 16);
}

// ------------------------------------------------------------------ row metadata of a pass
// mode 0: verify rows (node i of sequence b); mode 1: draft catch-up rows; mode 2: draft tree level.
__global__ void k_setup(int mode, const int32_t *ctx_len, TreeTables tt, RowMeta meta, int T,
                        int rows_per_seq, int m, int d, int n_exp, const double *inv_freq, int half) {
    const int r = blockIdx.x;
    const int b = r / rows_per_seq, i = r % rows_per_seq;
    const int C = ctx_len[b];
    int pos, slot, nvis, base, kv_end;
    uint64_t mask;
    if (mode == 0) {
        pos = C + tt.depth[i]; slot = C + i; nvis = C; base = C; mask = tt.anc_mask[i]; kv_end = C + T;
    } else if (mode == 1) {
        pos = C - m + i; slot = pos; nvis = pos + 1; base = 0; mask = 0; kv_end = C;
    } else {
        const int u = tt.level_nodes[d * 64 + i];
        pos = C - 1 + d; slot = C + tt.exp_index[u]; nvis = C; base = C; mask = tt.draft_mask[u];
        kv_end = C + n_exp;
    }
    if (threadIdx.x == 0) {
        meta.row_b[r] = b; meta.row_pos[r] = pos; meta.row_slot[r] = slot; meta.row_nvis[r] = nvis;
        meta.row_base[r] = base; meta.row_mask[r] = mask;
        if (i == 0) meta.kv_end[b] = kv_end;
    }
    for (int j = threadIdx.x; j < half; j += blockDim.x) {
        const double ang = (double)pos * inv_freq[j];
        meta.rope_cos[(size_t)r * half + j] = (float)cos(ang);
        meta.rope_sin[(size_t)r * half + j] = (float)sin(ang);
    }
}

// ------------------------------------------------------------------ embedding / fc input
template <typename WT>
__global__ void k_embed(const int32_t *tok, const WT *E, float *x, int H) {
    const int r = blockIdx.x;
    const size_t t = (size_t)tok[r];
    for (int j = threadIdx.x; j < H; j += blockDim.x) x[(size_t)r * H + j] = ldf(E, t * H + j);
}

template <typename WT>
__global__ void k_fc_input(const int32_t *tok, const WT *E, const float *feat, float *act, int H) {
    // grid (rows, chunks of the hidden dimension): few rows, so the columns supply the parallelism
    const int r = blockIdx.x;
    const size_t t = (size_t)tok[r];
    for (int j = blockIdx.y * blockDim.x + threadIdx.x; j < H; j += gridDim.y * blockDim.x) {
        act[(size_t)r * 2 * H + j] = ldf(E, t * H + j);
        act[(size_t)r * 2 * H + H + j] = feat[(size_t)r * H + j];
    }
}

template <typename WT>
__global__ void k_level_inputs(const int32_t *tree_tokens, const WT *E, const float *fhat,
                               const int32_t *level_nodes, const int32_t *parent, float *act,
                               int n_level, int T, int H) {
    const int r = blockIdx.x;
    const int b = r / n_level, u = level_nodes[r % n_level];
    const size_t t = (size_t)tree_tokens[b * T + u];
    const float *f = fhat + ((size_t)b * T + parent[u]) * H;
    for (int j = blockIdx.y * blockDim.x + threadIdx.x; j < H; j += gridDim.y * blockDim.x) {
        act[(size_t)r * 2 * H + j] = ldf(E, t * H + j);
        act[(size_t)r * 2 * H + H + j] = f[j];
    }
}

// ------------------------------------------------------------------ RMSNorm
template <typename WT>
__global__ __launch_bounds__(256) void k_rmsnorm(const float *x, const WT *g, float *out, int H, float eps) {
    __shared__ float red[4];
    const int r = blockIdx.x;
    const float *xr = x + (size_t)r * H;
    float ss = 0.f;
    for (int j = threadIdx.x; j < H; j += 256) { const float v = xr[j]; ss += v * v; }
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float inv = 1.0f / sqrtf(tot / (float)H + eps);
    for (int j = threadIdx.x; j < H; j += 256) out[(size_t)r * H + j] = xr[j] * inv * ldf(g, j);
}

// ------------------------------------------------------------------ generic GEMM: one wave per output column
template <typename WT, bool ACC>
__global__ __launch_bounds__(256) void k_gemm(const float *__restrict__ A, int lda, const WT *__restrict__ W,
                                              float *Y, int ldy, int M, int N, int K) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + wave;
    if (n >= N) return;
    const WT *wrow = W + (size_t)n * K;
    for (int m0 = 0; m0 < M; m0 += 8) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        for (int k = lane * 4; k < K; k += 256) {
            const float w0 = ldf(wrow, k), w1 = ldf(wrow, k + 1), w2 = ldf(wrow, k + 2), w3 = ldf(wrow, k + 3);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (m0 + i < M) {
                    const float4 a = *(const float4 *)(A + (size_t)(m0 + i) * lda + k);
                    acc[i] += a.x * w0 + a.y * w1 + a.z * w2 + a.w * w3;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float v = acc[i];
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
            if (lane == 0 && m0 + i < M) {
                float *y = Y + (size_t)(m0 + i) * ldy + n;
                *y = ACC ? (*y + v) : v;
            }
        }
    }
}

// ------------------------------------------------------------------ RoPE + KV append
template <typename CT>
__global__ void k_rope_append(const float *qkv, RowMeta meta, float *qrot, CT *kc, CT *vc, int H,
                              int n_heads, int DH, int cap) {
    const int r = blockIdx.x, h = blockIdx.y, i = threadIdx.x, half = DH / 2;
    const int b = meta.row_b[r], slot = meta.row_slot[r];
    const float c = meta.rope_cos[(size_t)r * half + i], s = meta.rope_sin[(size_t)r * half + i];
    const float *row = qkv + (size_t)r * 3 * H;
    const float q0 = row[h * DH + i], q1 = row[h * DH + half + i];
    const float k0 = row[H + h * DH + i], k1 = row[H + h * DH + half + i];
    const float v0 = row[2 * H + h * DH + i], v1 = row[2 * H + h * DH + half + i];
    qrot[(size_t)r * H + h * DH + i] = q0 * c - q1 * s;
    qrot[(size_t)r * H + h * DH + half + i] = q1 * c + q0 * s;
    const size_t o = (((size_t)b * n_heads + h) * cap + slot) * DH;
    stf(kc, o + i, k0 * c - k1 * s);
    stf(kc, o + half + i, k1 * c + k0 * s);
    stf(vc, o + i, v0);
    stf(vc, o + half + i, v1);
}

// ------------------------------------------------------------------ attention (split over the keys)
// grid (nsplit, n_heads, batch); 256 threads = 64 rows x 4 parts.
template <typename CT, int DH>
__global__ __launch_bounds__(256) void k_attn(const float *qrot, RowMeta meta, const CT *kc, const CT *vc,
                                              float *o_part, float *ml, int rows_per_seq, int n_heads,
                                              int cap, int nsplit, int H) {
    constexpr int KT = 32;
    __shared__ float sk[KT][DH + 1];
    __shared__ float sv[KT][DH];
    __shared__ float sp[64][KT + 1];
    const int s = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, t = tid >> 2, part = tid & 3;
    const int r = b * rows_per_seq + t;
    const bool row_ok = t < rows_per_seq;
    const float scale = rsqrtf((float)DH);
    float q[DH];
#pragma unroll
    for (int d = 0; d < DH; ++d) q[d] = row_ok ? qrot[(size_t)r * H + h * DH + d] * scale : 0.f;
    const int nvis = row_ok ? meta.row_nvis[r] : 0;
    const int base = row_ok ? meta.row_base[r] : 0;
    const uint64_t mask = row_ok ? meta.row_mask[r] : 0;
    const int kv_end = meta.kv_end[b];
    int chunk = (kv_end + nsplit - 1) / nsplit;
    chunk = (chunk + KT - 1) / KT * KT;
    const int j0 = s * chunk, j1 = min(kv_end, j0 + chunk);
    const CT *kb = kc + ((size_t)b * n_heads + h) * cap * DH;
    const CT *vb = vc + ((size_t)b * n_heads + h) * cap * DH;
    constexpr int DP = DH / 4;
    float acc[DP];
#pragma unroll
    for (int d = 0; d < DP; ++d) acc[d] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    for (int jt = j0; jt < j1; jt += KT) {
        __syncthreads();
        for (int e = tid; e < KT * DH; e += 256) {
            const int jj = e / DH, d = e % DH, j = jt + jj;
            const bool ok = j < j1;
            sk[jj][d] = ok ? ldf(kb, (size_t)j * DH + d) : 0.f;
            sv[jj][d] = ok ? ldf(vb, (size_t)j * DH + d) : 0.f;
        }
        __syncthreads();
        float sc[KT / 4];
        float tmax = -INFINITY;
#pragma unroll
        for (int i = 0; i < KT / 4; ++i) {
            const int jj = part + 4 * i, j = jt + jj;
            const int rel = j - base;
            const bool vis = row_ok && j < j1 &&
                             (j < nvis || (rel >= 0 && rel < 64 && ((mask >> rel) & 1ull)));
            float dot = 0.f;
#pragma unroll
            for (int d = 0; d < DH; ++d) dot += q[d] * sk[jj][d];
            sc[i] = vis ? dot : -INFINITY;
            tmax = fmaxf(tmax, sc[i]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 1));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 2));
        const float m_new = fmaxf(m_run, tmax);
        const float alpha = (m_run == -INFINITY) ? 0.f : __expf(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < KT / 4; ++i) {
            const float p = (sc[i] == -INFINITY) ? 0.f : __expf(sc[i] - m_new);
            sp[t][part + 4 * i] = p;
            psum += p;
        }
        psum += __shfl_xor(psum, 1);
        psum += __shfl_xor(psum, 2);
        l_run = l_run * alpha + psum;
        m_run = m_new;
        __syncthreads();
#pragma unroll
        for (int d = 0; d < DP; ++d) acc[d] *= alpha;
        for (int jj = 0; jj < KT; ++jj) {
            const float p = sp[t][jj];
#pragma unroll
            for (int d = 0; d < DP; ++d) acc[d] += p * sv[jj][part * DP + d];
        }
    }
    if (row_ok) {
        float *o = o_part + (((size_t)r * n_heads + h) * nsplit + s) * DH + part * DP;
#pragma unroll
        for (int d = 0; d < DP; ++d) o[d] = acc[d];
        if (part == 0) {
            float *p = ml + (((size_t)r * n_heads + h) * nsplit + s) * 2;
            p[0] = m_run;
            p[1] = l_run;
        }
    }
}

// merge the per-split partial results: grid (rows, n_heads), DH threads
__global__ void k_attn_combine(const float *o_part, const float *ml, float *out, int n_heads, int nsplit,
                               int DH, int H) {
    const int r = blockIdx.x, h = blockIdx.y, d = threadIdx.x;
    const float *p = ml + ((size_t)r * n_heads + h) * nsplit * 2;
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, p[2 * s]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float ms = p[2 * s];
        if (ms == -INFINITY) continue;
        const float w = __expf(ms - M);
        num += w * o_part[(((size_t)r * n_heads + h) * nsplit + s) * DH + d];
        den += w * p[2 * s + 1];
    }
    out[(size_t)r * H + h * DH + d] = num / den;
}

// ------------------------------------------------------------------ elementwise
__global__ void k_silu_mul(const float *gu, float *act, int F, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const size_t r = i / F, f = i % F;
    const float g = gu[r * 2 * F + 2 * f], u = gu[r * 2 * F + 2 * f + 1];
    act[i] = g / (1.0f + __expf(-g)) * u;
}

__global__ void k_resblock(float *x, const float *y, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float v = y[i];
    x[i] += v / (1.0f + __expf(-v));
}

__global__ void k_copy(float *dst, const float *src, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = src[i];
}

// ------------------------------------------------------------------ top-k of each row (k <= 16)
// Descending value, equal values ordered by ascending index; one block per row.
__global__ __launch_bounds__(256) void k_topk(const float *logits, int ld, int V, int k, int32_t *idx, float *val) {
    __shared__ float bv[256];
    __shared__ int bi[256];
    __shared__ int chosen[KOALA_TOPK_MAX];
    const int r = blockIdx.x, tid = threadIdx.x;
    const float *row = logits + (size_t)r * ld;
    for (int it = 0; it < k; ++it) {
        float best = -INFINITY;
        int besti = 0x7fffffff;
        for (int j = tid; j < V; j += 256) {
            bool taken = false;
            for (int c = 0; c < it; ++c) taken |= (chosen[c] == j);
            if (taken) continue;
            const float v = row[j];
            if (v > best || (v == best && j < besti) || besti == 0x7fffffff) { best = v; besti = j; }
        }
        bv[tid] = best;
        bi[tid] = besti;
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) {
            if (tid < o) {
                const float v2 = bv[tid + o];
                const int i2 = bi[tid + o];
                if (i2 != 0x7fffffff && (bi[tid] == 0x7fffffff || v2 > bv[tid] || (v2 == bv[tid] && i2 < bi[tid]))) {
                    bv[tid] = v2;
                    bi[tid] = i2;
                }
            }
            __syncthreads();
        }
        if (tid == 0) {
            chosen[it] = bi[0];
            idx[(size_t)r * k + it] = bi[0];
            if (val) val[(size_t)r * k + it] = bv[0];
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ draft bookkeeping
__global__ void k_gather_last(const float *x, float *dst, size_t dst_stride, int m, int H) {
    const int b = blockIdx.x;
    for (int j = threadIdx.x; j < H; j += blockDim.x)
        dst[(size_t)b * dst_stride + j] = x[((size_t)b * m + m - 1) * H + j];
}

__global__ void k_store_fhat(const float *x, float *fhat, const int32_t *level_nodes, int n_level, int T, int H) {
    const int r = blockIdx.x, b = r / n_level, u = level_nodes[r % n_level];
    for (int j = threadIdx.x; j < H; j += blockDim.x)
        fhat[((size_t)b * T + u) * H + j] = x[(size_t)r * H + j];
}

__global__ void k_set_root(const int32_t *tok_in, int m, int32_t *tree_tokens, float *scores, int batch, int T) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    tree_tokens[b * T] = tok_in[b * m + m - 1];
    if (scores) scores[b * T] = 0.f;
}

// children of the nodes of one level receive their parent's top-k tokens by rank
__global__ void k_fill_children(const int32_t *topk_idx, const float *topk_val, int kmax,
                                const int32_t *level_nodes, int n_level, TreeTables tt, int d,
                                int32_t *tree_tokens, float *scores, int batch, int T) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= batch * T) return;
    const int b = i / T, c = i % T;
    if (tt.depth[c] != d + 1) return;
    const int p = tt.parent[c];
    int li = -1;
    for (int j = 0; j < n_level; ++j)
        if (level_nodes[j] == p) li = j;
    if (li < 0) return;
    const size_t row = (size_t)b * n_level + li;
    tree_tokens[i] = topk_idx[row * kmax + tt.rank[c]];
    if (scores) scores[i] = topk_val[row * kmax + tt.rank[c]];
}

// Medusa: node of depth j, rank r receives head j's rank-r token; logits row = (j-1)*batch + b
__global__ void k_fill_medusa(const int32_t *topk_idx, const float *topk_val, int kmax, TreeTables tt,
                              int32_t *tree_tokens, float *scores, int batch, int T) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= batch * T) return;
    const int b = i / T, c = i % T;
    const int dj = tt.depth[c];
    if (dj == 0) return;
    const size_t row = (size_t)(dj - 1) * batch + b;
    tree_tokens[i] = topk_idx[row * kmax + tt.rank[c]];
    if (scores) scores[i] = topk_val[row * kmax + tt.rank[c]];
}

// ------------------------------------------------------------------ acceptance
__global__ void k_accept(TreeTables tt, int T, int D, const int32_t *tree_tokens, const int32_t *greedy,
                         int32_t *accept_len, int32_t *accept_path, int32_t *next_token, int batch) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    const int32_t *tok = tree_tokens + (size_t)b * T;
    const int32_t *g = greedy + (size_t)b * T;
    int32_t *path = accept_path + (size_t)b * (D + 1);
    int cur = 0, a = 0;
    path[0] = 0;
    for (;;) {
        int nxt = -1;
        for (int c = cur + 1; c < T; ++c) {
            if (tt.parent[c] == cur && tok[c] == g[cur]) { nxt = c; break; }
        }
        if (nxt < 0 || a >= D) break;
        cur = nxt;
        path[++a] = cur;
    }
    for (int j = a + 1; j <= D; ++j) path[j] = -1;
    accept_len[b] = a;
    next_token[b] = g[cur];
}

// Move the accepted nodes' rows to slots C..C+a.  Each thread owns one element column and
// walks the path in order, so a slot is always read before a later step overwrites it.
template <typename CT>
__global__ void k_kv_commit(CT *kc, CT *vc, const int32_t *ctx_len, const int32_t *accept_len,
                            const int32_t *accept_path, int D, int max_batch, int n_heads, int cap, int DH) {
    const int l = blockIdx.x, b = blockIdx.y, h = blockIdx.z, d = threadIdx.x;
    const int C = ctx_len[b], a = accept_len[b];
    const size_t base = ((((size_t)l * max_batch + b) * n_heads + h) * cap) * DH + d;
    for (int j = 1; j <= a; ++j) {
        const int node = accept_path[(size_t)b * (D + 1) + j];
        if (node == j) continue;
        kc[base + (size_t)(C + j) * DH] = kc[base + (size_t)(C + node) * DH];
        vc[base + (size_t)(C + j) * DH] = vc[base + (size_t)(C + node) * DH];
    }
}

__global__ void k_advance(int32_t *ctx_len, const int32_t *accept_len, int batch) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < batch) ctx_len[b] += accept_len[b] + 1;
}

// Inputs of the next draft step from one accepted path (one sequence): block i <= a copies the
// feature of path node i to row i and sets tok_next[i] to the token that follows it (the next
// path node's token, or the target's own token after the last accepted node); the same tokens are
// appended to out_tokens[n_done + i] while that index is below max_new.  grid D+1 blocks.
__global__ void k_gen_next(const float *feat_out, const int32_t *tree_tokens, const int32_t *accept_len,
                           const int32_t *accept_path, const int32_t *next_token, int T, int H, float *feat_next,
                           int32_t *tok_next, int32_t *out_tokens, int n_done, int max_new) {
    const int i = blockIdx.x, a = accept_len[0];
    if (i > a) return;
    const int node = accept_path[i];
    if (node < 0 || node >= T) return;   // never for a path the accept scan wrote
    const float *src = feat_out + (size_t)node * H;
    float *dst = feat_next + (size_t)i * H;
    for (int j = threadIdx.x; j < H; j += blockDim.x) dst[j] = src[j];
    if (threadIdx.x == 0) {
        int32_t tok = next_token[0];
        if (i < a) {
            const int nx = accept_path[i + 1];
            if (nx >= 0 && nx < T) tok = tree_tokens[nx];
        }
        tok_next[i] = tok;
        if (n_done + i < max_new) out_tokens[n_done + i] = tok;
    }
}

// Streaming read of n 16-byte words (measurement aid): every thread xors what it reads; the result is
// stored only to keep the loads alive.
typedef __attribute__((ext_vector_type(4))) unsigned int rd_u32x4;
__global__ __launch_bounds__(256) void k_stream_read(const rd_u32x4 *src, size_t n, unsigned *sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    rd_u32x4 acc = {0u, 0u, 0u, 0u};
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n; i += 4 * stride) {
        const rd_u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
        const rd_u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride);
        const rd_u32x4 d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < n; i += stride) acc ^= __builtin_nontemporal_load(src + i);
    const unsigned r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (r == 0x9e3779b9u) sink[0] = r;
}

inline int cdiv(size_t a, size_t b) { return (int)((a + b - 1) / b); }

}  // namespace

// =====================================================================================================
namespace kg {

static void setup(hipStream_t s, const koala_ctx *c, int mode, int batch, int rows_per_seq, int m, int d) {
    const int half = c->shape.head_dim / 2;
    const double *inv_freq = (const double *)(c->ws);  // first table of the workspace
    k_setup<<<batch * rows_per_seq, 64, 0, s>>>(mode, c->kv.ctx_len, c->tt, c->meta, c->T, rows_per_seq, m, d,
                                                c->n_exp, inv_freq, half);
}
void setup_verify(hipStream_t s, const koala_ctx *c, int batch) { setup(s, c, 0, batch, c->T, 0, 0); }
void setup_catchup(hipStream_t s, const koala_ctx *c, int batch, int m) { setup(s, c, 1, batch, m, m, 0); }
void setup_level(hipStream_t s, const koala_ctx *c, int batch, int d, int n_level) {
    setup(s, c, 2, batch, n_level, 0, d);
}

void embed_rows(hipStream_t s, bool bf16, const int32_t *tok, const void *E, float *x, int rows, int H) {
    if (bf16) k_embed<bf16_t><<<rows, 256, 0, s>>>(tok, (const bf16_t *)E, x, H);
    else k_embed<float><<<rows, 256, 0, s>>>(tok, (const float *)E, x, H);
}

void fc_input(hipStream_t s, bool bf16, const int32_t *tok, const void *E, const float *feat, float *act,
              int rows, int H) {
    const dim3 grid(rows, std::max(1, std::min(16, H / 256)));
    if (bf16) k_fc_input<bf16_t><<<grid, 256, 0, s>>>(tok, (const bf16_t *)E, feat, act, H);
    else k_fc_input<float><<<grid, 256, 0, s>>>(tok, (const float *)E, feat, act, H);
}

void level_inputs(hipStream_t s, bool bf16, const int32_t *tree_tokens, const void *E, const float *fhat,
                  const int32_t *level_nodes, const int32_t *parent, float *act, int batch, int n_level,
                  int T, int H) {
    const dim3 grid(batch * n_level, std::max(1, std::min(16, H / 256)));
    if (bf16)
        k_level_inputs<bf16_t><<<grid, 256, 0, s>>>(tree_tokens, (const bf16_t *)E, fhat, level_nodes, parent, act,
                                                    n_level, T, H);
    else
        k_level_inputs<float><<<grid, 256, 0, s>>>(tree_tokens, (const float *)E, fhat, level_nodes, parent, act,
                                                   n_level, T, H);
}

void rmsnorm(hipStream_t s, bool bf16, const float *x, const void *g, float *out, int rows, int H, float eps) {
    if (bf16) k_rmsnorm<bf16_t><<<rows, 256, 0, s>>>(x, (const bf16_t *)g, out, H, eps);
    else k_rmsnorm<float><<<rows, 256, 0, s>>>(x, (const float *)g, out, H, eps);
}

void gemm(hipStream_t s, bool bf16, const float *A, int lda, const void *W, float *Y, int ldy, int M, int N,
          int K, bool accumulate) {
    const dim3 grid(cdiv(N, 4));
    if (bf16) {
        if (accumulate) k_gemm<bf16_t, true><<<grid, 256, 0, s>>>(A, lda, (const bf16_t *)W, Y, ldy, M, N, K);
        else k_gemm<bf16_t, false><<<grid, 256, 0, s>>>(A, lda, (const bf16_t *)W, Y, ldy, M, N, K);
    } else {
        if (accumulate) k_gemm<float, true><<<grid, 256, 0, s>>>(A, lda, (const float *)W, Y, ldy, M, N, K);
        else k_gemm<float, false><<<grid, 256, 0, s>>>(A, lda, (const float *)W, Y, ldy, M, N, K);
    }
}

void rope_append(hipStream_t s, bool bf16, const float *qkv, const RowMeta &meta, float *qrot, void *kcache,
                 void *vcache, int rows, int H, int n_heads, int head_dim, int capacity, int) {
    const dim3 grid(rows, n_heads);
    if (bf16)
        k_rope_append<bf16_t><<<grid, head_dim / 2, 0, s>>>(qkv, meta, qrot, (bf16_t *)kcache, (bf16_t *)vcache, H,
                                                            n_heads, head_dim, capacity);
    else
        k_rope_append<float><<<grid, head_dim / 2, 0, s>>>(qkv, meta, qrot, (float *)kcache, (float *)vcache, H,
                                                           n_heads, head_dim, capacity);
}

void attention(hipStream_t s, bool bf16, const float *qrot, const RowMeta &meta, const void *kcache,
               const void *vcache, float *o_part, float *ml, float *attn_out, int batch, int rows_per_seq,
               int n_heads, int head_dim, int capacity, int nsplit) {
    const dim3 grid(nsplit, n_heads, batch);
    const int H = n_heads * head_dim;
#define KOALA_ATTN(CT, DHV)                                                                             \
    k_attn<CT, DHV><<<grid, 256, 0, s>>>(qrot, meta, (const CT *)kcache, (const CT *)vcache, o_part, ml, \
                                         rows_per_seq, n_heads, capacity, nsplit, H)
    if (head_dim == 128) {
        if (bf16) KOALA_ATTN(bf16_t, 128); else KOALA_ATTN(float, 128);
    } else {
        if (bf16) KOALA_ATTN(bf16_t, 64); else KOALA_ATTN(float, 64);
    }
#undef KOALA_ATTN
    if (attn_out)
        k_attn_combine<<<dim3(batch * rows_per_seq, n_heads), head_dim, 0, s>>>(o_part, ml, attn_out, n_heads,
                                                                               nsplit, head_dim, H);
}

void silu_mul(hipStream_t s, const float *gu, float *act, int rows, int F) {
    const size_t n = (size_t)rows * F;
    k_silu_mul<<<cdiv(n, 256), 256, 0, s>>>(gu, act, F, n);
}

void resblock_update(hipStream_t s, float *x, const float *y, int n) {
    k_resblock<<<cdiv(n, 256), 256, 0, s>>>(x, y, (size_t)n);
}

void copy_f32(hipStream_t s, float *dst, const float *src, size_t n) {
    k_copy<<<cdiv(n, 256), 256, 0, s>>>(dst, src, n);
}

void topk_rows(hipStream_t s, const float *logits, int ld, int rows, int V, int k, int32_t *idx, float *val) {
    k_topk<<<rows, 256, 0, s>>>(logits, ld, V, k, idx, val);
}

void store_fhat(hipStream_t s, const float *x, float *fhat, const int32_t *level_nodes, int batch, int n_level,
                int T, int H) {
    k_store_fhat<<<batch * n_level, 256, 0, s>>>(x, fhat, level_nodes, n_level, T, H);
}

void set_root(hipStream_t s, const int32_t *tok_in, int m, int32_t *tree_tokens, float *scores, int batch, int T) {
    k_set_root<<<cdiv(batch, 64), 64, 0, s>>>(tok_in, m, tree_tokens, scores, batch, T);
}

void fill_children(hipStream_t s, const int32_t *topk_idx, const float *topk_val, int kmax,
                   const int32_t *level_nodes, int n_level, const TreeTables &tt, int d, int32_t *tree_tokens,
                   float *scores, int batch, int T) {
    k_fill_children<<<cdiv((size_t)batch * T, 64), 64, 0, s>>>(topk_idx, topk_val, kmax, level_nodes, n_level, tt, d,
                                                              tree_tokens, scores, batch, T);
}

void fill_medusa(hipStream_t s, const int32_t *topk_idx, const float *topk_val, int kmax, const TreeTables &tt,
                 int32_t *tree_tokens, float *scores, int batch, int T, int) {
    k_fill_medusa<<<cdiv((size_t)batch * T, 64), 64, 0, s>>>(topk_idx, topk_val, kmax, tt, tree_tokens, scores,
                                                            batch, T);
}

void accept_scan(hipStream_t s, const TreeTables &tt, int T, int D, const int32_t *tree_tokens,
                 const int32_t *greedy, int32_t *accept_len, int32_t *accept_path, int32_t *next_token, int batch) {
    k_accept<<<cdiv(batch, 64), 64, 0, s>>>(tt, T, D, tree_tokens, greedy, accept_len, accept_path, next_token,
                                            batch);
}

void kv_commit(hipStream_t s, bool bf16, void *kcache, void *vcache, const int32_t *ctx_len,
               const int32_t *accept_len, const int32_t *accept_path, int D, int n_layers, int max_batch,
               int batch, int n_heads, int capacity, int head_dim) {
    const dim3 grid(n_layers, batch, n_heads);
    if (bf16)
        k_kv_commit<bf16_t><<<grid, head_dim, 0, s>>>((bf16_t *)kcache, (bf16_t *)vcache, ctx_len, accept_len,
                                                      accept_path, D, max_batch, n_heads, capacity, head_dim);
    else
        k_kv_commit<float><<<grid, head_dim, 0, s>>>((float *)kcache, (float *)vcache, ctx_len, accept_len,
                                                     accept_path, D, max_batch, n_heads, capacity, head_dim);
}

void advance_ctx(hipStream_t s, int32_t *ctx_len, const int32_t *accept_len, int batch) {
    k_advance<<<cdiv(batch, 64), 64, 0, s>>>(ctx_len, accept_len, batch);
}

// dst[b * dst_stride + j] = x[(b*m + m-1) * H + j]: the newest row of every sequence
void gather_last_rows(hipStream_t s, const float *x, float *dst, size_t dst_stride, int batch, int m, int H) {
    k_gather_last<<<batch, 256, 0, s>>>(x, dst, dst_stride, m, H);
}

void stream_read(hipStream_t s, const void *src, size_t bytes, unsigned *sink) {
    k_stream_read<<<2048, 256, 0, s>>>((const rd_u32x4 *)src, bytes / 16, sink);
}

void gen_next(hipStream_t s, const float *feat_out, const int32_t *tree_tokens, const int32_t *accept_len,
              const int32_t *accept_path, const int32_t *next_token, int T, int D, int H, float *feat_next,
              int32_t *tok_next, int32_t *out_tokens, int n_done, int max_new) {
    k_gen_next<<<D + 1, 256, 0, s>>>(feat_out, tree_tokens, accept_len, accept_path, next_token, T, H, feat_next,
                                     tok_next, out_tokens, n_done, max_new);
}

}  // namespace kg
