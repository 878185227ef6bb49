// Non-greedy (temperature) drafting and acceptance, section 2.2:
//   * children of a tree node are draws without replacement from softmax(draft logits / temperature);
//   * the acceptance walk keeps child x with probability min(1, q(x)/d(x)); after a rejection the target
//     distribution becomes norm(max(0, q - d)), the rejected token leaves the draft distribution, and the
//     next child (in draw order) is tried; where the walk stops, one token is drawn from what q has become.
// Every uniform random number is an input.  One workgroup of 1024 threads per row / sequence.
//
// A draw is an inverse CDF over ascending token id: the first id at which the running sum of the weights
// exceeds u * total.  The vocabulary is cut into segments of 256 consecutive ids; a wave sums a segment
// with lane l holding ids 4l..4l+3 (fp64, fixed shuffle order), the segment sums are added in id order, and
// inside the chosen segment a wave-wide inclusive scan in lane order finds the id.  All orders are fixed,
// so a draw does not depend on scheduling.
#include "koala_internal.h"

namespace {

constexpr int NT = 1024;         // threads per workgroup
constexpr int NW = NT / 64;      // waves per workgroup
constexpr int SEG = 256;          // ids per segment
constexpr int MAX_SEG = 1024;     // vocabularies up to 262144
constexpr int UNR = 4;            // independent loads in flight per thread in the vocabulary-wide passes

struct Shared {
    double seg[MAX_SEG];
    double red[NW];
    float fmax_[NW];
    double total, base, target;
    int sidx, idx, fallback;
    int kids[64];
    int nk;
};

__device__ __forceinline__ double wave_sum(double v) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// every thread gets the sum of v over the workgroup (waves added in order)
__device__ __forceinline__ double block_sum(double v, Shared &sh) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
    for (int k = 0; k < NW; ++k) t += sh.red[k];
    return t;
}

__device__ __forceinline__ float block_max(float v, Shared &sh) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.fmax_[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = sh.fmax_[0];
    for (int k = 1; k < NW; ++k) t = fmaxf(t, sh.fmax_[k]);
    return t;
}

// the four weights of lane l in segment s (zero past V)
__device__ __forceinline__ void seg_load(const float *w, int V, int s, int l, float *x) {
    const int i = s * SEG + 4 * l;
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = i + e < V ? w[i + e] : 0.f;
}

__device__ __forceinline__ double seg_lane_sum(const float *x) {
    return (((double)x[0] + (double)x[1]) + (double)x[2]) + (double)x[3];
}

// sh.seg[s] = sum of w over segment s, for all segments (wave k takes segments k, k+NW, ...)
__device__ void segment_sums(const float *w, int V, Shared &sh) {
    const int wave = threadIdx.x >> 6, l = threadIdx.x & 63, nseg = (V + SEG - 1) / SEG;
    __syncthreads();
    for (int s0 = wave; s0 < nseg; s0 += 4 * NW) {   // four segments' loads in flight per wave
        float x[4][4];
#pragma unroll
        for (int k = 0; k < 4; ++k) seg_load(w, V, s0 + NW * k, l, x[k]);   // past the last segment: zeros
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const double t = wave_sum(seg_lane_sum(x[k]));
            if (l == 0 && s0 + NW * k < nseg) sh.seg[s0 + NW * k] = t;
        }
    }
    __syncthreads();
}

// Index of the first id at which the running sum of w exceeds u * sum(w); the last positive id if rounding
// leaves none; 0 if nothing is positive.  sh.seg must hold the segment sums of w.  Every thread gets it.
__device__ int block_inverse_cdf(const float *w, int V, double u, Shared &sh) {
    const int tid = threadIdx.x, nseg = (V + SEG - 1) / SEG;
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
        for (int s = 0; s < nseg; ++s) total += sh.seg[s];
        const double target = u * total;
        double run = 0.0;
        int t = -1;
        for (int s = 0; s < nseg; ++s) {
            if (run + sh.seg[s] > target) { t = s; break; }
            run += sh.seg[s];
        }
        sh.fallback = 0;
        if (t < 0) {   // rounding: the last segment that holds anything
            sh.fallback = 1;
            for (int s = nseg - 1; s >= 0; --s)
                if (sh.seg[s] > 0.0) { t = s; break; }
        }
        sh.sidx = t;
        sh.base = run;
        sh.target = target;
        sh.idx = 0;
    }
    __syncthreads();
    if (tid < 64 && sh.sidx >= 0) {   // wave 0 resolves the id inside the segment
        const int s = sh.sidx, l = tid;
        float x[4];
        seg_load(w, V, s, l, x);
        const double own = seg_lane_sum(x);
        double incl = own;
        for (int o = 1; o < 64; o <<= 1) {
            const double t = __shfl_up(incl, o);
            if (l >= o) incl += t;
        }
        const double lo = sh.base + (incl - own), hi = sh.base + incl;
        int pick = -1, lastpos = -1;
        double run = lo;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (x[e] > 0.f) {
                lastpos = s * SEG + 4 * l + e;
                run += (double)x[e];
                if (pick < 0 && run > sh.target) pick = lastpos;
            }
        }
        const bool mine = !sh.fallback && lo <= sh.target && hi > sh.target && pick >= 0;
        // the first lane that claims the id wins; otherwise the last positive id of the segment
        const unsigned long long claims = __ballot(mine);
        int last_all = lastpos;
        for (int o = 32; o > 0; o >>= 1) last_all = max(last_all, __shfl_xor(last_all, o));
        if (claims) {
            const int first = __ffsll((long long)claims) - 1;
            const int got = __shfl(pick, first);
            if (l == 0) sh.idx = got;
        } else if (l == 0) {
            sh.idx = last_all < 0 ? 0 : last_all;
        }
    }
    __syncthreads();
    return sh.idx;
}

// children of node p in draw order (ascending rank, then node id) into sh.kids
__device__ void list_children(const TreeTables &tt, int T, int p, Shared &sh) {
    __syncthreads();
    if (threadIdx.x == 0) {
        int n = 0;
        for (int c = 0; c < T && n < 64; ++c) {
            if (tt.parent[c] != p) continue;
            int j = n++;
            while (j > 0 && tt.rank[sh.kids[j - 1]] > tt.rank[c]) { sh.kids[j] = sh.kids[j - 1]; --j; }
            sh.kids[j] = c;
        }
        sh.nk = n;
    }
    __syncthreads();
}

// w[i] = exp((z[i] - max z) / tau); returns sum(w).  z and w may alias.  copy: optional copy of z.
__device__ double softmax_weights(const float *z, float *w, float *copy, int V, float inv_tau, Shared &sh) {
    const int tid = threadIdx.x;
    float m = -INFINITY;
    for (int i0 = tid; i0 < V; i0 += NT * UNR) {
        float v[UNR];
#pragma unroll
        for (int k = 0; k < UNR; ++k) v[k] = i0 + k * NT < V ? z[i0 + k * NT] : -INFINITY;
#pragma unroll
        for (int k = 0; k < UNR; ++k) {
            m = fmaxf(m, v[k]);
            if (copy && i0 + k * NT < V) copy[i0 + k * NT] = v[k];
        }
    }
    m = block_max(m, sh);
    double s = 0.0;
    for (int i0 = tid; i0 < V; i0 += NT * UNR) {
        float v[UNR];
#pragma unroll
        for (int k = 0; k < UNR; ++k) v[k] = i0 + k * NT < V ? z[i0 + k * NT] : -INFINITY;
#pragma unroll
        for (int k = 0; k < UNR; ++k) {
            if (i0 + k * NT < V) {
                const float e = expf((v[k] - m) * inv_tau);
                w[i0 + k * NT] = e;
                s += (double)e;
            }
        }
    }
    return block_sum(s, sh);
}

// w[i] /= total over the vocabulary
__device__ void scale_by(float *w, int V, double total) {
    for (int i0 = threadIdx.x; i0 < V; i0 += NT * UNR) {
        float v[UNR];
#pragma unroll
        for (int k = 0; k < UNR; ++k) v[k] = i0 + k * NT < V ? w[i0 + k * NT] : 0.f;
#pragma unroll
        for (int k = 0; k < UNR; ++k)
            if (i0 + k * NT < V) w[i0 + k * NT] = (float)((double)v[k] / total);
    }
}

// dst row (b * n_level + li) = src row (src_row0 + b), for every li: the shared per-depth logits of a
// Medusa-style head get one private copy per parent node.  grid: batch * n_level.
__global__ __launch_bounds__(256) void k_repeat_rows(const float *src, int src_row0, float *dst, int V, int n_level) {
    const int row = blockIdx.x, b = row / n_level;
    const float *s = src + (size_t)(src_row0 + b) * V;
    float *d = dst + (size_t)row * V;
    for (int i = threadIdx.x; i < V; i += 256) d[i] = s[i];
}

// grid: batch * n_level rows.  z: [rows][V] draft logits of the level's nodes (overwritten by weights).
__global__ __launch_bounds__(NT) void k_sample_children(float *z, const int32_t *level_nodes, int n_level,
                                                         TreeTables tt, int T, int V, float inv_tau,
                                                         const float *u_draw, int32_t *tree_tokens,
                                                         float *draft_logits) {
    __shared__ Shared sh;
    const int row = blockIdx.x, b = row / n_level, li = row % n_level, tid = threadIdx.x;
    const int p = level_nodes[li];
    if (p < 0 || p >= T) return;   // uniform; never for tables the host built
    list_children(tt, T, p, sh);
    float *zr = z + (size_t)row * V;
    (void)softmax_weights(zr, zr, draft_logits + ((size_t)b * T + p) * V, V, inv_tau, sh);
    segment_sums(zr, V, sh);
    for (int j = 0; j < sh.nk; ++j) {
        const int c = sh.kids[j];
        const int idx = block_inverse_cdf(zr, V, (double)u_draw[(size_t)b * T + c], sh);
        if (tid == 0) {
            tree_tokens[(size_t)b * T + c] = idx;
            zr[idx] = 0.f;   // drawn without replacement
        }
        __syncthreads();
        if (tid < 64) {      // wave 0 refreshes the sum of the segment that lost the token
            const int s = idx / SEG;
            float x[4];
            seg_load(zr, V, s, tid, x);
            const double t = wave_sum(seg_lane_sum(x));
            if (tid == 0) sh.seg[s] = t;
        }
        __syncthreads();
    }
}

// grid: batch.  qv, dv: [batch][V] scratch.
__global__ __launch_bounds__(NT) void k_accept_sample(TreeTables tt, int T, int D, int V, float inv_tau,
                                                       const int32_t *tree_tokens, const float *target_logits,
                                                       const float *draft_logits, const float *u_accept,
                                                       const float *u_resample, float *qv_all, float *dv_all,
                                                       int32_t *accept_len, int32_t *accept_path,
                                                       int32_t *next_token) {
    __shared__ Shared sh;
    const int b = blockIdx.x, tid = threadIdx.x;
    float *qv = qv_all + (size_t)b * V, *dv = dv_all + (size_t)b * V;
    const int32_t *tok = tree_tokens + (size_t)b * T;
    int32_t *path = accept_path + (size_t)b * (D + 1);
    int cur = 0, a = 0;
    if (tid == 0) path[0] = 0;
    for (;;) {
        // q = softmax(target logits at cur)
        double tot = softmax_weights(target_logits + ((size_t)b * T + cur) * V, qv, nullptr, V, inv_tau, sh);
        scale_by(qv, V, tot);
        list_children(tt, T, cur, sh);
        const int nk = a < D ? sh.nk : 0;
        bool moved = false;
        if (nk > 0) {
            tot = softmax_weights(draft_logits + ((size_t)b * T + cur) * V, dv, nullptr, V, inv_tau, sh);
            scale_by(dv, V, tot);
            __syncthreads();
            for (int j = 0; j < nk; ++j) {
                const int c = sh.kids[j];
                int x = tok[c];
                x = x < 0 ? 0 : x >= V ? V - 1 : x;
                const double qx = (double)qv[x], dx = (double)dv[x];
                const double ratio = dx > 0.0 ? fmin(1.0, qx / dx) : 0.0;
                if (dx > 0.0 && (double)u_accept[(size_t)b * T + c] < ratio) {
                    cur = c;
                    ++a;
                    if (tid == 0) path[a] = c;
                    moved = true;
                    break;
                }
                // rejected: q <- norm(max(0, q - d)) (kept if that is all zero); d loses x and is renormalised
                double rs = 0.0, ds = 0.0;
                for (int i0 = tid; i0 < V; i0 += NT * UNR) {
                    float qa[UNR], da[UNR];
#pragma unroll
                    for (int k = 0; k < UNR; ++k) {
                        const bool in = i0 + k * NT < V;
                        qa[k] = in ? qv[i0 + k * NT] : 0.f;
                        da[k] = in ? dv[i0 + k * NT] : 0.f;
                    }
#pragma unroll
                    for (int k = 0; k < UNR; ++k) {
                        rs += (double)fmaxf(0.f, qa[k] - da[k]);
                        if (i0 + k * NT != x) ds += (double)da[k];
                    }
                }
                const double R = block_sum(rs, sh);
                const double Dn = block_sum(ds, sh);
                for (int i0 = tid; i0 < V; i0 += NT * UNR) {
                    float qa[UNR], da[UNR];
#pragma unroll
                    for (int k = 0; k < UNR; ++k) {
                        const bool in = i0 + k * NT < V;
                        qa[k] = in ? qv[i0 + k * NT] : 0.f;
                        da[k] = in ? dv[i0 + k * NT] : 0.f;
                    }
#pragma unroll
                    for (int k = 0; k < UNR; ++k) {
                        const int i = i0 + k * NT;
                        if (i < V) {
                            if (R > 0.0) qv[i] = (float)((double)fmaxf(0.f, qa[k] - da[k]) / R);
                            dv[i] = (i == x) ? 0.f : (Dn > 0.0 ? (float)((double)da[k] / Dn) : da[k]);
                        }
                    }
                }
                __syncthreads();
            }
        }
        if (!moved) {
            segment_sums(qv, V, sh);
            const int idx = block_inverse_cdf(qv, V, (double)u_resample[(size_t)b * T + cur], sh);
            if (tid == 0) {
                next_token[b] = idx;
                accept_len[b] = a;
                for (int j = a + 1; j <= D; ++j) path[j] = -1;
            }
            return;
        }
        __syncthreads();
    }
}

}  // namespace

namespace ks {

int max_vocab() { return MAX_SEG * SEG; }

void repeat_rows(hipStream_t st, const float *src, int src_row0, float *dst, int V, int n_level, int batch) {
    k_repeat_rows<<<batch * n_level, 256, 0, st>>>(src, src_row0, dst, V, n_level);
}

void sample_children(hipStream_t st, float *logits, const int32_t *level_nodes, int n_level, const TreeTables &tt,
                     int T, int V, float temperature, const float *u_draw, int32_t *tree_tokens,
                     float *draft_logits, int batch) {
    k_sample_children<<<batch * n_level, NT, 0, st>>>(logits, level_nodes, n_level, tt, T, V, 1.0f / temperature,
                                                      u_draw, tree_tokens, draft_logits);
}

void accept_sample(hipStream_t st, const TreeTables &tt, int T, int D, int V, float temperature,
                   const int32_t *tree_tokens, const float *target_logits, const float *draft_logits,
                   const float *u_accept, const float *u_resample, float *qv, float *dv, int32_t *accept_len,
                   int32_t *accept_path, int32_t *next_token, int batch) {
    k_accept_sample<<<batch, NT, 0, st>>>(tt, T, D, V, 1.0f / temperature, tree_tokens, target_logits, draft_logits,
                                          u_accept, u_resample, qv, dv, accept_len, accept_path, next_token);
}

}  // namespace ks
