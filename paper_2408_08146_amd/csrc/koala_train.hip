// Adversarial training step of a draft head (section 3.2, Algorithm 1, Eq. 5 and 6) in fp32: the
// discriminator's forward and backward passes with its gradient-descent update, the draft-head loss and its
// gradient at the logits, and the forward pass / backward pass / update of a Medusa-style head.  Dense
// products run on the fp32 matrix pipe (16x16x4 MFMA); everything else is small row-wise kernels.
#include <math.h>

#include "koala_internal.h"

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;

// ---------------------------------------------------------------------------------------------
// C[M,N] = alpha * sum_k A(m,k) B(k,n) + beta * C[m,n]; A(m,k) = A[m*sam + k*sak], B(k,n) = B[k*sbk + n*sbn],
// C row-major with leading dimension ldc.  Workgroup = 4 waves on a 64 x 64 tile, each wave 32 x 32 as 2 x 2
// MFMA tiles, K in chunks of 16 through LDS.  MFMA 16x16x4 operands: lane (i = l%16, k = l/16) holds A[i][k]
// and B[k][i]; the result lane holds C[4*(l/16) + r][l%16], r = 0..3.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_sgemm(const float *__restrict__ A, long sam, long sak,
                                               const float *__restrict__ B, long sbk, long sbn, float *C, long ldc,
                                               int M, int N, int K, float alpha, float beta) {
    constexpr int LD = 17;
    __shared__ float As[64 * LD], Bs[64 * LD];   // As[m][k], Bs[n][k]
    const int tid = threadIdx.x, wave = tid >> 6, l = tid & 63, li = l & 15, lk = l >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64, wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
    f32x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < K; k0 += 16) {
        // 64 x 16 elements of each operand: 4 per thread; the faster-varying index follows the smaller stride
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tid + 256 * i;
            const int ma = sak <= sam ? e / 16 : e % 64, ka = sak <= sam ? e % 16 : e / 64;
            As[ma * LD + ka] = (m0 + ma < M && k0 + ka < K) ? A[(long)(m0 + ma) * sam + (long)(k0 + ka) * sak] : 0.f;
            const int nb = sbk <= sbn ? e / 16 : e % 64, kb = sbk <= sbn ? e % 16 : e / 64;
            Bs[nb * LD + kb] = (n0 + nb < N && k0 + kb < K) ? B[(long)(k0 + kb) * sbk + (long)(n0 + nb) * sbn] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            float a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = As[(wm + 16 * i + li) * LD + 4 * kk + lk];
                b[i] = Bs[(wn + 16 * i + li) * LD + 4 * kk + lk];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + wm + 16 * i + 4 * lk + r, n = n0 + wn + 16 * j + li;
                if (m < M && n < N) {
                    float *c = C + (long)m * ldc + n;
                    *c = alpha * acc[i][j][r] + (beta != 0.f ? beta * *c : 0.f);
                }
            }
}

void sgemm(hipStream_t st, const float *A, long sam, long sak, const float *B, long sbk, long sbn, float *C, long ldc,
           int M, int N, int K, float alpha, float beta) {
    k_sgemm<<<dim3((N + 63) / 64, (M + 63) / 64), 256, 0, st>>>(A, sam, sak, B, sbk, sbn, C, ldc, M, N, K, alpha, beta);
}

__device__ __forceinline__ float softplus(float x) { return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x))); }
__device__ __forceinline__ float sigmoidf(float x) { return 1.0f / (1.0f + expf(-x)); }

// sum over the workgroup (256 threads); every thread gets the total
__device__ __forceinline__ float block_sum(float v, float *sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}
__device__ __forceinline__ float block_max(float v, float *sh) {
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}

// u[r][v] = z[r % n][v] + (r < n ? la : lb)[r % n][v]: the mapped hidden state joined to a logits row
__global__ void k_join(const float *z, const float *la, const float *lb, float *u, int n, int V, int rows) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long)rows * V) return;
    const int r = (int)(i / V), v = (int)(i % V), p = r % n;
    u[i] = z[(long)p * V + v] + (r < n ? la : lb)[(long)p * V + v];
}

// y += bias (kept as the pre-activation), a = max(y, 0)
__global__ void k_bias_relu(float *y, const float *bias, float *a, int rows, int W) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long)rows * W) return;
    const float v = y[i] + bias[i % W];
    y[i] = v;
    a[i] = fmaxf(v, 0.f);
}

// g[r][j] *= (pre[r][j] > 0)
__global__ void k_relu_back(float *g, const float *pre, long n) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n && !(pre[i] > 0.f)) g[i] = 0.f;
}

// bias[j] -= lr * sum_r g[r][j]
__global__ void k_bias_update(float *bias, const float *g, int rows, int W, float lr) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= W) return;
    float t = 0.f;
    for (int r = 0; r < rows; ++r) t += g[(long)r * W + j];
    bias[j] -= lr * t;
}

// Scores s (pre-sigmoid, the last layer's bias already added) -> dL/ds per row and the loss.  One workgroup.
//   mode 0 (Eq. 6): rows [0, n) are the draft's, [n, 2n) the target's:
//          L_D = mean softplus(s_d) + mean softplus(-s_q);  ds_d = sigmoid(s)/n, ds_q = -(1 - sigmoid(s))/n
//   mode 1 (Eq. 5, adversarial term): n draft rows: L = lambda mean softplus(-s); ds = -lambda (1 - sigmoid(s))/n
__global__ __launch_bounds__(256) void k_score_loss(const float *s, const float *bias_p, float *ds, float *loss, int n,
                                                    int mode, float lambda) {
    __shared__ float sh[4];
    const float bias = bias_p[0];
    float part = 0.f;
    const int rows = mode == 0 ? 2 * n : n;
    for (int r = threadIdx.x; r < rows; r += 256) {
        const float v = s[r] + bias;
        if (mode == 0) {
            part += r < n ? softplus(v) : softplus(-v);
            ds[r] = r < n ? sigmoidf(v) / n : -(1.0f - sigmoidf(v)) / n;
        } else {
            part += lambda * softplus(-v);
            ds[r] = -lambda * (1.0f - sigmoidf(v)) / n;
        }
    }
    const float tot = block_sum(part, sh);
    if (threadIdx.x == 0) loss[0] = tot / n;
}

// g[r][j] = ds[r] * w[j]   (backward of the width-1 layer towards its input)
__global__ void k_outer(const float *ds, const float *w, float *g, int rows, int W) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long)rows * W) return;
    g[i] = ds[i / W] * w[i % W];
}

// gz[p][v] = gu[p][v] + gu[n + p][v]
__global__ void k_fold_rows(const float *gu, float *gz, int n, int V) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (long)n * V) gz[i] = gu[i] + gu[(long)n * V + i];
}

// Distillation term (cross-entropy of softmax(d) against softmax(q)) of one row per workgroup:
// ce[r] = lse(d) - sum_v softmax(q)_v d_v, and grad[r][v] (+)= (softmax(d)_v - softmax(q)_v) / n
__global__ __launch_bounds__(256) void k_distill(const float *q, const float *d, float *grad, float *ce, int V, int n,
                                                 int accumulate) {
    __shared__ float sh[4];
    const int r = blockIdx.x;
    const float *qr = q + (long)r * V, *dr = d + (long)r * V;
    float mq = -INFINITY, md = -INFINITY;
    for (int v = threadIdx.x; v < V; v += 256) { mq = fmaxf(mq, qr[v]); md = fmaxf(md, dr[v]); }
    mq = block_max(mq, sh);
    md = block_max(md, sh);
    float sq = 0.f, sd = 0.f, qd = 0.f;
    for (int v = threadIdx.x; v < V; v += 256) {
        const float eq = expf(qr[v] - mq);
        sq += eq;
        sd += expf(dr[v] - md);
        qd += eq * dr[v];
    }
    sq = block_sum(sq, sh);
    sd = block_sum(sd, sh);
    qd = block_sum(qd, sh);
    if (threadIdx.x == 0) ce[r] = (md + logf(sd)) - qd / sq;
    float *gr = grad + (long)r * V;
    for (int v = threadIdx.x; v < V; v += 256) {
        const float g = (expf(dr[v] - md) / sd - expf(qr[v] - mq) / sq) / n;
        gr[v] = accumulate ? gr[v] + g : g;
    }
}

// loss[0] = mean of ce[0..n)
__global__ __launch_bounds__(256) void k_mean(const float *ce, float *loss, int n) {
    __shared__ float sh[4];
    float t = 0.f;
    for (int r = threadIdx.x; r < n; r += 256) t += ce[r];
    t = block_sum(t, sh);
    if (threadIdx.x == 0) loss[0] = t / n;
}

// x_next = x + SiLU(y)
__global__ void k_res_silu(const float *x, const float *y, float *xn, long n) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) xn[i] = x[i] + y[i] / (1.0f + expf(-y[i]));
}

// gy = gx * SiLU'(y)
__global__ void k_silu_back(const float *gx, const float *y, float *gy, long n) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float s = 1.0f / (1.0f + expf(-y[i]));
    gy[i] = gx[i] * s * (1.0f + y[i] * (1.0f - s));
}

inline int blocks(long n) { return (int)((n + 255) / 256); }
inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }

struct DiscWs {
    float *z, *u, *ds, *s, *ce;
    float *a[3], *pre[3], *g[3];   // a[k]: input of FC layer k (a[0] = u); pre[k]: its output before ReLU; g: gradients
    size_t bytes;
};

// rows = 2n for the discriminator step (draft rows, then target rows), n for the draft-head gradient
DiscWs carve_disc(const koala_disc_shape &s, int n, char *base) {
    DiscWs w{};
    size_t off = 0;
    auto take = [&](size_t floats) {
        float *p = base ? (float *)(base + off) : nullptr;
        off += up256(floats * sizeof(float));
        return p;
    };
    const int rows = 2 * n, V = s.vocab, Dh = s.fc_hidden;
    w.z = take((size_t)n * V);
    w.u = take((size_t)rows * V);
    w.ds = take(rows);
    w.s = take(rows);
    w.ce = take(n);
    w.a[0] = w.u;
    w.g[0] = take((size_t)rows * V);
    for (int k = 1; k < s.n_fc; ++k) {
        w.pre[k - 1] = take((size_t)rows * Dh);
        w.a[k] = take((size_t)rows * Dh);
        w.g[k] = take((size_t)rows * Dh);
    }
    w.bytes = off;
    return w;
}

bool shape_ok(const koala_disc_shape *s) {
    return s && s->hidden > 0 && s->vocab > 0 && s->n_fc >= 1 && s->n_fc <= 3 && (s->n_fc == 1 || s->fc_hidden > 0);
}
bool params_ok(const koala_disc_shape *s, const koala_disc_params *p) {
    if (!p || !p->w_lin) return false;
    for (int k = 0; k < s->n_fc; ++k)
        if (!p->w_fc[k] || !p->b_fc[k]) return false;
    return true;
}
inline int fc_in(const koala_disc_shape &s, int k) { return k == 0 ? s.vocab : s.fc_hidden; }
inline int fc_out(const koala_disc_shape &s, int k) { return k == s.n_fc - 1 ? 1 : s.fc_hidden; }

// scores of `rows` joined rows u: leaves every layer's input and pre-activation in the workspace, s = w_last . a
void disc_forward(hipStream_t st, const koala_disc_shape &s, const koala_disc_params &p, const DiscWs &w, int rows) {
    for (int k = 0; k < s.n_fc; ++k) {
        const int in = fc_in(s, k), out = fc_out(s, k);
        if (k == s.n_fc - 1) {   // width 1: s[r] = a[r] . w (bias added where the score is used)
            sgemm(st, w.a[k], in, 1, p.w_fc[k], 1, in, w.s, 1, rows, 1, in, 1.f, 0.f);
        } else {
            sgemm(st, w.a[k], in, 1, p.w_fc[k], 1, in, w.pre[k], out, rows, out, in, 1.f, 0.f);
            k_bias_relu<<<blocks((long)rows * out), 256, 0, st>>>(w.pre[k], p.b_fc[k], w.a[k + 1], rows, out);
        }
    }
}

// from ds (dL/ds per row) back to g[0] = dL/du; lr > 0: the parameters are updated on the way (each layer's
// input gradient is taken with the layer's old weights first)
void disc_backward(hipStream_t st, const koala_disc_shape &s, const koala_disc_params &p, const DiscWs &w, int rows,
                   float lr) {
    for (int k = s.n_fc - 1; k >= 0; --k) {
        const int in = fc_in(s, k), out = fc_out(s, k);
        const float *gout = k == s.n_fc - 1 ? w.ds : w.g[k + 1];   // dL/d(pre of layer k): [rows, out]
        if (k == s.n_fc - 1) k_outer<<<blocks((long)rows * in), 256, 0, st>>>(w.ds, p.w_fc[k], w.g[k], rows, in);
        else sgemm(st, gout, out, 1, p.w_fc[k], in, 1, w.g[k], in, rows, in, out, 1.f, 0.f);
        if (lr > 0.f) {
            // W_k[out, in] -= lr * gout^T a_k ;  b_k -= lr * column sums of gout
            sgemm(st, gout, 1, out, w.a[k], in, 1, p.w_fc[k], in, out, in, rows, -lr, 1.f);
            k_bias_update<<<blocks(out), 256, 0, st>>>(p.b_fc[k], gout, rows, out, lr);
        }
        if (k > 0) k_relu_back<<<blocks((long)rows * in), 256, 0, st>>>(w.g[k], w.pre[k - 1], (long)rows * in);
    }
}

}  // namespace

extern "C" {

koala_status koala_train_workspace_bytes(const koala_disc_shape *shape, int n_rows, size_t *out) {
    if (!shape || !out) return KOALA_E_NULL;
    if (!shape_ok(shape) || n_rows < 1) return KOALA_E_SHAPE;
    *out = carve_disc(*shape, n_rows, nullptr).bytes;
    return KOALA_OK;
}

koala_status koala_train_disc_step(const koala_disc_shape *shape, const koala_disc_params *params, void *hip_stream,
                                   int n_rows, const float *h, const float *q_logits, const float *d_logits, float lr,
                                   void *workspace, size_t workspace_bytes, float *loss_out) {
    if (!shape || !params || !h || !q_logits || !d_logits || !workspace || !loss_out) return KOALA_E_NULL;
    if (!shape_ok(shape) || n_rows < 1 || !(lr >= 0.f)) return KOALA_E_SHAPE;
    if (!params_ok(shape, params)) return KOALA_E_NULL;
    const koala_disc_shape &s = *shape;
    const DiscWs w = carve_disc(s, n_rows, (char *)workspace);
    if (workspace_bytes < w.bytes) return KOALA_E_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    const int n = n_rows, V = s.vocab, H = s.hidden, rows = 2 * n;
    // z = h W_lin^T, u = [z + d ; z + q]
    sgemm(st, h, H, 1, params->w_lin, 1, H, w.z, V, n, V, H, 1.f, 0.f);
    k_join<<<blocks((long)rows * V), 256, 0, st>>>(w.z, d_logits, q_logits, w.u, n, V, rows);
    disc_forward(st, s, *params, w, rows);
    k_score_loss<<<1, 256, 0, st>>>(w.s, params->b_fc[s.n_fc - 1], w.ds, loss_out, n, 0, 0.f);
    disc_backward(st, s, *params, w, rows, lr);
    if (lr > 0.f) {
        // u = W_lin h + logits for both halves: dL/dW_lin = (g_u[draft rows] + g_u[target rows])^T h
        k_fold_rows<<<blocks((long)n * V), 256, 0, st>>>(w.g[0], w.z, n, V);
        sgemm(st, w.z, 1, V, h, H, 1, params->w_lin, H, V, H, n, -lr, 1.f);
    }
    return hipGetLastError() == hipSuccess ? KOALA_OK : KOALA_E_DEVICE;
}

koala_status koala_train_gen_grad(const koala_disc_shape *shape, const koala_disc_params *params, void *hip_stream,
                                  int n_rows, const float *h, const float *q_logits, const float *d_logits,
                                  float lambda, void *workspace, size_t workspace_bytes, float *loss_out,
                                  float *grad_d) {
    if (!shape || !params || !h || !q_logits || !d_logits || !workspace || !loss_out || !grad_d) return KOALA_E_NULL;
    if (!shape_ok(shape) || n_rows < 1 || !(lambda >= 0.f)) return KOALA_E_SHAPE;
    if (!params_ok(shape, params)) return KOALA_E_NULL;
    const koala_disc_shape &s = *shape;
    const DiscWs w = carve_disc(s, n_rows, (char *)workspace);
    if (workspace_bytes < w.bytes) return KOALA_E_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    const int n = n_rows, V = s.vocab, H = s.hidden;
    sgemm(st, h, H, 1, params->w_lin, 1, H, w.z, V, n, V, H, 1.f, 0.f);
    k_join<<<blocks((long)n * V), 256, 0, st>>>(w.z, d_logits, d_logits, w.u, n, V, n);
    disc_forward(st, s, *params, w, n);
    k_score_loss<<<1, 256, 0, st>>>(w.s, params->b_fc[s.n_fc - 1], w.ds, loss_out, n, 1, lambda);
    disc_backward(st, s, *params, w, n, 0.f);
    // dL_G/dd = dL_adv/du (u = z + d) + the distillation term's gradient
    if (hipMemcpyAsync(grad_d, w.g[0], (size_t)n * V * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess)
        return KOALA_E_DEVICE;
    k_distill<<<n, 256, 0, st>>>(q_logits, d_logits, grad_d, w.ce, V, n, 1);
    k_mean<<<1, 256, 0, st>>>(w.ce, loss_out + 1, n);
    return hipGetLastError() == hipSuccess ? KOALA_OK : KOALA_E_DEVICE;
}

koala_status koala_train_medusa_workspace_bytes(int n_rows, int hidden, int K, size_t *out) {
    if (!out) return KOALA_E_NULL;
    if (n_rows < 1 || hidden < 1 || K < 1 || K > 8) return KOALA_E_SHAPE;
    // x_0 .. x_K, y_0 .. y_{K-1}, gx, gx', gy
    *out = up256((size_t)n_rows * hidden * sizeof(float)) * (size_t)(2 * K + 4);
    return KOALA_OK;
}

static void medusa_forward(hipStream_t st, int n, int H, int K, float *const *blocks_w, const float *h, float *xs,
                           float *ys, size_t stride) {
    (void)hipMemcpyAsync(xs, h, (size_t)n * H * sizeof(float), hipMemcpyDeviceToDevice, st);
    for (int k = 0; k < K; ++k) {
        float *x = xs + stride * k, *y = ys + stride * k;
        sgemm(st, x, H, 1, blocks_w[k], 1, H, y, H, n, H, H, 1.f, 0.f);
        k_res_silu<<<blocks((long)n * H), 256, 0, st>>>(x, y, xs + stride * (k + 1), (long)n * H);
    }
}

koala_status koala_train_medusa_head_forward(void *hip_stream, int n_rows, int hidden, int vocab, int K,
                                             float *const *blocks_w, const float *w_lm, const float *h,
                                             void *workspace, size_t workspace_bytes, float *d_logits) {
    if (!blocks_w || !w_lm || !h || !workspace || !d_logits) return KOALA_E_NULL;
    size_t need = 0;
    if (koala_train_medusa_workspace_bytes(n_rows, hidden, K, &need) != KOALA_OK || vocab < 1) return KOALA_E_SHAPE;
    if (workspace_bytes < need) return KOALA_E_WORKSPACE;
    for (int k = 0; k < K; ++k)
        if (!blocks_w[k]) return KOALA_E_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t stride = up256((size_t)n_rows * hidden * sizeof(float)) / sizeof(float);
    float *xs = (float *)workspace, *ys = xs + stride * (K + 1);
    medusa_forward(st, n_rows, hidden, K, blocks_w, h, xs, ys, stride);
    sgemm(st, xs + stride * K, hidden, 1, w_lm, 1, hidden, d_logits, vocab, n_rows, vocab, hidden, 1.f, 0.f);
    return hipGetLastError() == hipSuccess ? KOALA_OK : KOALA_E_DEVICE;
}

koala_status koala_train_medusa_head_step(void *hip_stream, int n_rows, int hidden, int vocab, int K,
                                          float *const *blocks_w, const float *w_lm, const float *h,
                                          const float *grad_d, float lr, void *workspace, size_t workspace_bytes) {
    if (!blocks_w || !w_lm || !h || !grad_d || !workspace) return KOALA_E_NULL;
    size_t need = 0;
    if (koala_train_medusa_workspace_bytes(n_rows, hidden, K, &need) != KOALA_OK || vocab < 1 || !(lr >= 0.f))
        return KOALA_E_SHAPE;
    if (workspace_bytes < need) return KOALA_E_WORKSPACE;
    for (int k = 0; k < K; ++k)
        if (!blocks_w[k]) return KOALA_E_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    const int n = n_rows, H = hidden, V = vocab;
    const size_t stride = up256((size_t)n * H * sizeof(float)) / sizeof(float);
    float *xs = (float *)workspace, *ys = xs + stride * (K + 1), *gx = ys + stride * K, *gx2 = gx + stride,
          *gy = gx2 + stride;
    medusa_forward(st, n, H, K, blocks_w, h, xs, ys, stride);
    sgemm(st, grad_d, V, 1, w_lm, H, 1, gx, H, n, H, V, 1.f, 0.f);                 // gx = grad_d W_lm
    for (int k = K - 1; k >= 0; --k) {
        k_silu_back<<<blocks((long)n * H), 256, 0, st>>>(gx, ys + stride * k, gy, (long)n * H);
        // gx <- gx + gy W_k with the block's old weights, then W_k -= lr * gy^T x_k
        (void)hipMemcpyAsync(gx2, gx, (size_t)n * H * sizeof(float), hipMemcpyDeviceToDevice, st);
        sgemm(st, gy, H, 1, blocks_w[k], H, 1, gx2, H, n, H, H, 1.f, 1.f);
        sgemm(st, gy, 1, H, xs + stride * k, H, 1, blocks_w[k], H, H, H, n, -lr, 1.f);
        float *t = gx; gx = gx2; gx2 = t;
    }
    return hipGetLastError() == hipSuccess ? KOALA_OK : KOALA_E_DEVICE;
}

}  // extern "C"
