// Non-greedy (temperature) drafting and acceptance, section 2.2:
//   * children of a tree node are draws without replacement from softmax(draft logits / temperature);
//   * the acceptance walk keeps child x with probability min(1, q(x)/d(x)); after a rejection the target
//     distribution becomes norm(max(0, q - d)), the rejected token leaves the draft distribution, and the
//     next child (in draw order) is tried; where the walk stops, one token is drawn from what q has become.
// Every uniform random number is an input.  One workgroup of 256 threads per row / sequence; sums that
// decide a token are accumulated in double in a fixed order (thread t owns the contiguous index range
// [t*CH, (t+1)*CH), ranges are added in order of t), so results do not depend on scheduling.
#include "koala_internal.h"

namespace {

constexpr int NT = 256;

struct Shared {
    double part[NT];
    double total, base, target;
    float fmax_[4];
    float rowmax;
    int chunk, idx, fallback;
    int kids[64];
    int nk;
};

__device__ __forceinline__ float block_max(float v, Shared &sh) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.fmax_[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(sh.fmax_[0], sh.fmax_[1]), fmaxf(sh.fmax_[2], sh.fmax_[3]));
}

// sum of sh.part[0..NT) in index order; every thread gets it
__device__ __forceinline__ double block_total(Shared &sh) {
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int i = 0; i < NT; ++i) t += sh.part[i];
        sh.total = t;
    }
    __syncthreads();
    return sh.total;
}

// Index of the first element at which the running sum of w[0..V) exceeds u * sum(w); the last positive
// element if rounding leaves none; 0 if nothing is positive.  sh.part must hold the chunk sums of w.
__device__ int block_inverse_cdf(const float *w, int V, int CH, double u, Shared &sh) {
    const int tid = threadIdx.x;
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
        for (int i = 0; i < NT; ++i) total += sh.part[i];
        const double target = u * total;
        double run = 0.0;
        int t = -1;
        for (int i = 0; i < NT; ++i) {
            if (run + sh.part[i] > target) { t = i; break; }
            run += sh.part[i];
        }
        sh.fallback = 0;
        if (t < 0) {   // rounding: take the last chunk that holds anything
            sh.fallback = 1;
            for (int i = NT - 1; i >= 0; --i)
                if (sh.part[i] > 0.0) { t = i; break; }
        }
        sh.chunk = t;
        sh.base = run;
        sh.target = target;
        sh.idx = 0;
    }
    __syncthreads();
    if (tid == sh.chunk) {
        const int i0 = tid * CH, i1 = min(V, i0 + CH);
        double run = sh.base;
        int pick = -1, lastpos = -1;
        for (int i = i0; i < i1; ++i) {
            const float wi = w[i];
            if (wi > 0.f) {
                lastpos = i;
                run += (double)wi;
                if (pick < 0 && !sh.fallback && run > sh.target) pick = i;
            }
        }
        if (pick < 0) pick = lastpos;
        sh.idx = pick < 0 ? 0 : pick;
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

// w[i] = exp((z[i] - max z) / tau) written to w, chunk sums to sh.part.  z and w may alias.
__device__ void softmax_weights(const float *z, float *w, int V, int CH, float inv_tau, Shared &sh) {
    const int tid = threadIdx.x;
    float m = -INFINITY;
    for (int i = tid; i < V; i += NT) m = fmaxf(m, z[i]);
    m = block_max(m, sh);
    const int i0 = tid * CH, i1 = min(V, i0 + CH);
    double s = 0.0;
    for (int i = i0; i < i1; ++i) {
        const float e = expf((z[i] - m) * inv_tau);
        w[i] = e;
        s += (double)e;
    }
    sh.part[tid] = s;
    __syncthreads();
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
    float *out = draft_logits + ((size_t)b * T + p) * V;
    for (int i = tid; i < V; i += NT) out[i] = zr[i];
    __syncthreads();
    const int CH = (V + NT - 1) / NT;
    softmax_weights(zr, zr, V, CH, inv_tau, sh);
    for (int j = 0; j < sh.nk; ++j) {
        const int c = sh.kids[j];
        const double u = (double)u_draw[(size_t)b * T + c];
        const int idx = block_inverse_cdf(zr, V, CH, u, sh);
        if (tid == 0) tree_tokens[(size_t)b * T + c] = idx;
        if (tid == idx / CH) {   // owner removes the token and recomputes its chunk sum
            zr[idx] = 0.f;
            const int i0 = tid * CH, i1 = min(V, i0 + CH);
            double s = 0.0;
            for (int i = i0; i < i1; ++i) s += (double)zr[i];
            sh.part[tid] = s;
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
    const int CH = (V + NT - 1) / NT, i0 = tid * CH, i1 = min(V, i0 + CH);
    float *qv = qv_all + (size_t)b * V, *dv = dv_all + (size_t)b * V;
    const int32_t *tok = tree_tokens + (size_t)b * T;
    int32_t *path = accept_path + (size_t)b * (D + 1);
    int cur = 0, a = 0;
    if (tid == 0) path[0] = 0;
    for (;;) {
        // q = softmax(target logits at cur)
        softmax_weights(target_logits + ((size_t)b * T + cur) * V, qv, V, CH, inv_tau, sh);
        double tot = block_total(sh);
        for (int i = i0; i < i1; ++i) qv[i] = (float)((double)qv[i] / tot);
        __syncthreads();
        list_children(tt, T, cur, sh);
        const int nk = a < D ? sh.nk : 0;
        bool moved = false;
        if (nk > 0) {
            softmax_weights(draft_logits + ((size_t)b * T + cur) * V, dv, V, CH, inv_tau, sh);
            tot = block_total(sh);
            for (int i = i0; i < i1; ++i) dv[i] = (float)((double)dv[i] / tot);
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
                for (int i = i0; i < i1; ++i) {
                    rs += (double)fmaxf(0.f, qv[i] - dv[i]);
                    if (i != x) ds += (double)dv[i];
                }
                __syncthreads();
                sh.part[tid] = rs;
                const double R = block_total(sh);
                __syncthreads();
                sh.part[tid] = ds;
                const double Dn = block_total(sh);
                for (int i = i0; i < i1; ++i) {
                    if (R > 0.0) qv[i] = (float)((double)fmaxf(0.f, qv[i] - dv[i]) / R);
                    dv[i] = (i == x) ? 0.f : (Dn > 0.0 ? (float)((double)dv[i] / Dn) : dv[i]);
                }
                __syncthreads();
            }
        }
        if (!moved) {
            double s = 0.0;
            for (int i = i0; i < i1; ++i) s += (double)qv[i];
            __syncthreads();
            sh.part[tid] = s;
            const int idx = block_inverse_cdf(qv, V, CH, (double)u_resample[(size_t)b * T + cur], sh);
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
