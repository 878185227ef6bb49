// All decoder layers of one verification pass in a single cooperative kernel (bf16 path, one sequence,
// at most 32 rows).  Opt-in (KOALA_PERSISTENT=1): on the 7B shape it runs as fast as the per-layer kernels,
// not faster; the measurements that explain why are kept with the design notes.
//
// Why: with one kernel per step a layer costs ten dependent launches, and every weight-streaming GEMM starts
// with an empty memory pipeline and ends with a drain.  Here one workgroup per CU stays resident for the whole
// stack and its eight waves split into two roles:
//   * waves 0-3 ("stream" waves) do nothing but load weight tiles (64 rows x 64 k, 8 KiB, fragment-major) into
//     a ring of NS register slots and multiply them with activation tiles that wait in LDS.  Per projection
//     they first fill all NS slots (as soon as the chain waves allow it: right after this workgroup arrived at
//     the barrier that ends the previous projection, so that the tiles travel while the small step between the
//     two projections runs), then compute and reload slot by slot.  Loads of one wave return in order, so a
//     wave with a deep weight queue cannot also do latency-critical loads; hence the second role;
//   * waves 4-7 ("chain" waves) run everything on the dependency chain: they copy activation tiles from
//     global memory into the LDS ring, write the stream waves' partial sums out, execute the small steps
//     (fold + RMSNorm gain, RoPE + KV append, tree attention, split merge, SwiGLU) and meet the other
//     workgroups at a grid barrier after every step.
// Work is cut stream-K style: the (row group, k tile) pairs of a matrix are dealt out in equal contiguous
// ranges, so every workgroup streams the same number of bytes; a row group's partial sums land in one slot
// per contributing workgroup and are added by the consumer in slot order (deterministic).
//
// Memory safety: every global access of activations, partial sums, weights and caches goes through buffer
// instructions whose descriptors carry the exact allocation size, so an index error reads zeros or drops a
// store instead of faulting.  Data that one workgroup writes and another reads inside the kernel is written
// and read at agent scope (sc1), which needs no cache flushes.  Every wait is bounded; a timeout raises the
// abort flag, everything drains, and the host reports an error.
#include "koala_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef unsigned short __attribute__((may_alias)) u16_alias;
typedef unsigned long long __attribute__((may_alias)) u64_lds;

#ifndef KOALA_PL_NS
#define KOALA_PL_NS 4
#endif
constexpr int NS = KOALA_PL_NS;       // weight tiles a stream wave keeps in registers / in flight (3..6)
constexpr int XR = 8;                 // activation tiles in the LDS ring
constexpr int AUX_SC1 = 16, AUX_NT = 2;
constexpr int AUX_X = AUX_SC1;   // activation tiles: written by other workgroups inside the kernel
constexpr int MAX_LAYERS = 96;        // layers the weight address table in LDS holds
constexpr long long TIMEOUT_TICKS = 25000000LL;   // 0.25 s of the 100 MHz wall clock

__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f2bf(float v) {
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ rsrc_t make_rsrc(const void *p, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
// the cache policy is an immediate of the instruction, hence a template parameter
template <int AUX>
__device__ __forceinline__ u32x4 ld128(rsrc_t r, unsigned off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, AUX);
}
template <int AUX>
__device__ __forceinline__ f32x4 ldf4(rsrc_t r, unsigned off) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, AUX));
}
template <int AUX>
__device__ __forceinline__ float ldf1(rsrc_t r, unsigned off) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, AUX));
}
__device__ __forceinline__ void st128(rsrc_t r, unsigned off, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)off, 0, AUX_SC1);
}
__device__ __forceinline__ void stf4(rsrc_t r, unsigned off, f32x4 v) { st128(r, off, __builtin_bit_cast(u32x4, v)); }
__device__ __forceinline__ void stf1(rsrc_t r, unsigned off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, (int)off, 0, AUX_SC1);
}
__device__ __forceinline__ void st16(rsrc_t r, unsigned off, uint32_t v) {
    __builtin_amdgcn_raw_buffer_store_b16((unsigned short)v, r, (int)off, 0, AUX_SC1);
}

#define RFL(x) __builtin_amdgcn_readfirstlane(x)
#define LDS_LD(p) RFL(__hip_atomic_load((p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP))
#define LDS_ST(p, v) __hip_atomic_store((p), (v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)
#define LDS_RELEASE() __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local")
#define LDS_ACQUIRE() __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local")

// The four projections of a layer in execution order.
enum { G_QKV = 0, G_O = 1, G_GU = 2, G_DOWN = 3 };

// Stream-K geometry of one projection for this workgroup (ints only; kept in LDS).
struct Kind {
    int nrb;      // 64-row blocks (Npad / 64)
    int KT;       // 64-wide k tiles
    int total;    // (row groups of 4 blocks) * KT
    int geff;     // workgroups that get tiles
    int Npad;
    int t0, n;    // this workgroup's tile range [t0, t0 + n)
    int pad_;
};

struct __attribute__((aligned(16))) Ctl {
    Kind kind[4];
    int xflag[XR];    // xflag[s] = seq + 1 of the activation tile in ring slot s
    int done[4];      // tiles finished by stream wave w (monotonic)
    int p_ready[4];   // flushes staged by stream wave w
    int p_taken[4];   // flushes written out by chain wave w
    int cbar;         // chain-wave barrier counter
    int gbar;         // grid barrier generation reached
    int abort_l;
    int go;           // projections (counted from the first layer) whose first weight loads may be issued
};

__device__ __forceinline__ int sk_start(int w, int total, int geff) {
    return w >= geff ? total : (int)(((unsigned)w * (unsigned)total) / (unsigned)geff);   // host checks the range
}
// the workgroup whose range contains tile T
__device__ __forceinline__ int sk_owner(int T, int total, int geff) {
    return (int)((((unsigned)(T + 1) * (unsigned)geff) + (unsigned)total - 1u) / (unsigned)total) - 1;
}
// number of partial-sum slots of row group rg
__device__ __forceinline__ int sk_slots(int rg, const Kind &k) {
    return sk_owner((rg + 1) * k.KT - 1, k.total, k.geff) - sk_owner(rg * k.KT, k.total, k.geff) + 1;
}

// LDS of a workgroup (dynamic, above the 64 KiB a static allocation may have): the activation ring and the
// partial-sum staging (the attention step reuses both), then the control block and the weight addresses.
constexpr int AREA_BYTES = XR * 2 * 4096 + 4 * 2 * 4096;   // sized for MT = 2
struct Shared {
    unsigned char area[AREA_BYTES];
    Ctl ctl;
    // weight addresses (low, high word) of phase g = 4 * layer + projection: the stream waves read them from
    // here, because a global load in their instruction stream would have to wait for the whole weight queue
    unsigned wtab[MAX_LAYERS * 4][2];
    unsigned ltab[MAX_LAYERS * 4][2];   // per layer: input norm gain, post-attention norm gain, key cache, value cache
#ifdef KOALA_PL_TW
    long long tl[64][4];
#endif
};

// ---------------------------------------------------------------------------------------------
// helpers of the chain waves
// ---------------------------------------------------------------------------------------------
struct Chain {
    const kp::Params &p;
    Ctl *ctl;
    int c, l, w, G;            // chain wave 0..3, lane, workgroup, grid size
    unsigned long long gen;    // grid barrier generation
    unsigned long long shard_target;   // arrivals a shard counter shows when the current barrier is complete
    int cgen;                  // chain barrier generation
    bool dead;
};

__device__ void chain_sync(Chain &k) {
    ++k.cgen;
    if (k.l == 0) {
        __hip_atomic_fetch_add(&k.ctl->cbar, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        const long long tb = wall_clock64();
        while (LDS_LD(&k.ctl->cbar) < 4 * k.cgen) {
            __builtin_amdgcn_s_sleep(1);
            if (LDS_LD(&k.ctl->abort_l) || wall_clock64() - tb > TIMEOUT_TICKS) { LDS_ST(&k.ctl->abort_l, 1); break; }
        }
    }
    LDS_ACQUIRE();
}

// Grid barrier.  `all`: every workgroup arrives; otherwise only the first p.nclean workgroups (those that run the
// small steps) arrive and the others just wait for them.  Arriving means: all global stores of this workgroup's
// chain waves are complete.  go_after > 0: once the arrival is on its way, the stream waves of this workgroup
// may issue the first loads of projections < go_after.  Ordering matters here, because the memory pipeline of a
// CU serves its requests in issue order: whatever is issued after a burst of weight loads waits for the burst.
__device__ void grid_barrier(Chain &k, bool all, int go_after) {
    const bool tracer = k.p.trace && k.w == 0 && k.c == 0 && k.l == 0;
    const int ntr = 2 + 10 * k.p.L;
    const bool arrives = all || k.w < k.p.nclean;
    if (tracer) k.p.trace[ntr + (k.gen + 1 - k.p.bar_base)] = wall_clock64();         // work of the step issued

    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    if (tracer) k.p.trace[2 * ntr + (k.gen + 1 - k.p.bar_base)] = wall_clock64();     // stores acknowledged
    LDS_RELEASE();
    chain_sync(k);
    ++k.gen;
    k.shard_target += (unsigned long long)((all ? k.G : k.p.nclean) / 8);
    if (k.c == 0) {
        if (k.l == 0) {
            unsigned long long *bar = k.p.bar;
            const unsigned shard = k.w & 7;
            unsigned long long old = 0;
            if (arrives) old = __hip_atomic_fetch_add(bar + shard * 16, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (go_after > 0) LDS_ST(&k.ctl->go, go_after);
            if (arrives && old + 1 == k.shard_target)
                __hip_atomic_fetch_add(bar + 8 * 16, 1ULL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const long long tb = wall_clock64();
            while (__hip_atomic_load(bar + 8 * 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < k.gen * 8) {
                __builtin_amdgcn_s_sleep(1);
                if (__hip_atomic_load(k.p.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                    LDS_ST(&k.ctl->abort_l, 1);
                    break;
                }
                if (wall_clock64() - tb > TIMEOUT_TICKS) {
                    __hip_atomic_store(k.p.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    LDS_ST(&k.ctl->abort_l, 1);
                    break;
                }
            }
            LDS_ST(&k.ctl->gbar, (int)(k.gen & 0x7fffffff));
        }
    } else if (k.l == 0) {
        const long long tb = wall_clock64();
        while (LDS_LD(&k.ctl->gbar) != (int)(k.gen & 0x7fffffff)) {
            __builtin_amdgcn_s_sleep(1);
            if (LDS_LD(&k.ctl->abort_l) || wall_clock64() - tb > TIMEOUT_TICKS) { LDS_ST(&k.ctl->abort_l, 1); break; }
        }
    }
    LDS_ACQUIRE();
    if (tracer) k.p.trace[k.gen - k.p.bar_base] = wall_clock64();
    if (LDS_LD(&k.ctl->abort_l)) {
        // tell the workgroups that still wait at a barrier
        if (k.l == 0) __hip_atomic_store(k.p.abort_flag, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        k.dead = true;
    }
}

// Loads of partial sums are issued in deep batches with unconditional instructions: a slot that does not
// exist gets an offset past the end of the buffer, which reads zeros without touching memory.  A sum then
// costs one memory round trip per batch instead of one per slot; the order of the additions is fixed.
constexpr unsigned OOB = 0xFFFFFF00u;

// NV consecutive float4 (col % 4 == 0) of row m summed over the slots of the columns' row group; 2 * NB slots
// per round trip (two arrays, because one of twice the size is not kept in registers)
template <int NV, int NB>
__device__ __forceinline__ void psumv(rsrc_t rP, int Mp, const Kind &kd, int m, int col, f32x4 *out) {
    const int S = sk_slots(col >> 8, kd);
    const unsigned stride = (unsigned)Mp * (unsigned)kd.Npad * 4u;
    const unsigned base = ((unsigned)m * (unsigned)kd.Npad + (unsigned)col) * 4u;
#pragma unroll
    for (int i = 0; i < NV; ++i) out[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < S; s0 += 2 * NB) {
        f32x4 ta[NB][NV], tb[NB][NV];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const unsigned off = s0 + u < S ? base + (unsigned)(s0 + u) * stride : OOB;
#pragma unroll
            for (int i = 0; i < NV; ++i) ta[u][i] = ldf4<AUX_SC1>(rP, off + 16u * i);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const unsigned off = s0 + NB + u < S ? base + (unsigned)(s0 + NB + u) * stride : OOB;
#pragma unroll
            for (int i = 0; i < NV; ++i) tb[u][i] = ldf4<AUX_SC1>(rP, off + 16u * i);
        }
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int i = 0; i < NV; ++i) out[i] += ta[u][i];
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int i = 0; i < NV; ++i) out[i] += tb[u][i];
    }
}

// NC single columns of row m, all in the same row group as cols[0]
template <int NC, int NB>
__device__ __forceinline__ void psumc(rsrc_t rP, int Mp, const Kind &kd, int m, const int *cols, float *out) {
    const unsigned stride = (unsigned)Mp * (unsigned)kd.Npad * 4u;
#pragma unroll
    for (int i = 0; i < NC; ++i) out[i] = 0.f;
    int S[NC];
    int Smax = 0;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        S[i] = sk_slots(cols[i] >> 8, kd);
        Smax = max(Smax, S[i]);
    }
    for (int s0 = 0; s0 < Smax; s0 += NB) {
        float t[NB][NC];
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                const unsigned off = s0 + u < S[i]
                                         ? ((unsigned)m * (unsigned)kd.Npad + (unsigned)cols[i]) * 4u + (unsigned)(s0 + u) * stride
                                         : OOB;
                t[u][i] = ldf1<AUX_SC1>(rP, off);
            }
#pragma unroll
        for (int u = 0; u < NB; ++u)
#pragma unroll
            for (int i = 0; i < NC; ++i) out[i] += t[u][i];
    }
}

// 8 consecutive k of row m (k0 % 8 == 0) as hi/lo fragments
template <int MT>
__device__ __forceinline__ void store_frag8(rsrc_t rX, int m, int k0, const float *y) {
    uint32_t hi[8], lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        hi[e] = f2bf(y[e]);
        lo[e] = f2bf(y[e] - bf2f(hi[e]));
    }
    const int ks = k0 >> 5, lane = (m & 15) + 16 * ((k0 & 31) >> 3), mt = m >> 4;
    u32x4 h, q;
    h.x = hi[0] | (hi[1] << 16); h.y = hi[2] | (hi[3] << 16); h.z = hi[4] | (hi[5] << 16); h.w = hi[6] | (hi[7] << 16);
    q.x = lo[0] | (lo[1] << 16); q.y = lo[2] | (lo[3] << 16); q.z = lo[4] | (lo[5] << 16); q.w = lo[6] | (lo[7] << 16);
    const unsigned o = (unsigned)((((size_t)(ks * MT + mt) * 2) * 64 + lane) * 16);
    st128(rX, o, h);
    st128(rX, o + 64 * 16, q);
}

// 1 / sqrt(mean(x^2) + eps) of row m from the per-512-column sums of squares.  The loads are issued by
// the constructor and consumed by get(), so that they share a round trip with whatever is loaded in between.
struct RowScale {
    float t[16];
    float rest;
    __device__ __forceinline__ RowScale(rsrc_t rS, int nparts, int srows, int m) {
#pragma unroll
        for (int c = 0; c < 16; ++c) t[c] = ldf1<AUX_SC1>(rS, c < nparts ? (unsigned)(c * srows + m) * 4u : OOB);
        rest = 0.f;
        for (int c = 16; c < nparts; ++c) rest += ldf1<AUX_SC1>(rS, (unsigned)(c * srows + m) * 4u);
    }
    __device__ __forceinline__ float get(int H, float eps) const {
        float tot = rest;
#pragma unroll
        for (int c = 0; c < 16; ++c) tot += t[c];
        return 1.0f / sqrtf(tot / (float)H + eps);
    }
};

// ---------------------------------------------------------------------------------------------
// the small steps, executed by the chain waves of all workgroups; unit = one wave
// ---------------------------------------------------------------------------------------------
// x (+)= partial sums of `prev` (mode 1) or x as is (mode 0); optionally fragments of gain * x and the
// per-chunk sums of squares.  units: (512-column chunk, row)
template <int MT>
__device__ void step_fold(Chain &k, int mode, const Kind &prev, const void *gain, bool frags) {
    const kp::Params &p = k.p;
    const rsrc_t rx = make_rsrc(p.x, p.x_bytes), rP = make_rsrc(p.part, p.part_bytes);
    const rsrc_t rX = make_rsrc(p.Xf, p.xf_bytes), rS = make_rsrc(p.sums, p.sums_bytes);
    const rsrc_t rg = make_rsrc(gain, gain ? (unsigned)p.H * 2 : 0);
    const int nch = (p.H + 511) / 512;
    for (int u = k.w * 4 + k.c; u < nch * p.rows && k.w < p.nclean; u += p.nclean * 4) {
        const int c = u % nch, m = u / nch, j = (c * 64 + k.l) * 8;
        float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (j < p.H) {
            const unsigned xo = (unsigned)(((size_t)m * p.H + j) * 4);
            const f32x4 a = ldf4<AUX_SC1>(rx, xo), b = ldf4<AUX_SC1>(rx, xo + 16);
            const u32x4 g = ld128<0>(rg, frags ? (unsigned)j * 2 : OOB);
            if (mode != 0) {
                f32x4 ps[2];
                psumv<2, 10>(rP, MT * 16, prev, m, j, ps);
                v[0] = ps[0][0]; v[1] = ps[0][1]; v[2] = ps[0][2]; v[3] = ps[0][3];
                v[4] = ps[1][0]; v[5] = ps[1][1]; v[6] = ps[1][2]; v[7] = ps[1][3];
            }
            v[0] += a[0]; v[1] += a[1]; v[2] += a[2]; v[3] += a[3];
            v[4] += b[0]; v[5] += b[1]; v[6] += b[2]; v[7] += b[3];
            if (mode != 0) {
                stf4(rx, xo, (f32x4){v[0], v[1], v[2], v[3]});
                stf4(rx, xo + 16, (f32x4){v[4], v[5], v[6], v[7]});
            }
            if (frags) {
                const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
                float y[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) y[e] = v[e] * bf2f((e & 1) ? (gw[e >> 1] >> 16) : (gw[e >> 1] & 0xFFFFu));
                store_frag8<MT>(rX, m, j, y);
            }
        }
        if (frags) {
            float ss = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
            for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
            if (k.l == 0) stf1(rS, (unsigned)(((size_t)c * p.srows + m) * 4), ss);
        }
    }
}

// RoPE + KV append from the QKV partial sums.  units: (row, head); lane = pair index (head_dim 128)
template <int MT>
__device__ void step_rope(Chain &k, const Kind &kq, rsrc_t rK, rsrc_t rV) {
    const kp::Params &p = k.p;
    const rsrc_t rP = make_rsrc(p.part, p.part_bytes), rS = make_rsrc(p.sums, p.sums_bytes);
    const rsrc_t rq = make_rsrc(p.qrot, p.qrot_bytes);
    const int H = p.H, DH = 128, half = 64, i = k.l;
    for (int u = k.w * 4 + k.c; u < p.rows * p.n_heads && k.w < p.nclean; u += p.nclean * 4) {
        const int r = u / p.n_heads, h = u % p.n_heads;
        const int b = p.meta.row_b[r], slot = p.meta.row_slot[r];
        const float cs = p.meta.rope_cos[(size_t)r * half + i], sn = p.meta.rope_sin[(size_t)r * half + i];
        const int c0 = h * DH + i;
        const RowScale rsc(rS, (H + 511) / 512, p.srows, r);
        const int cols[6] = {c0, c0 + half, H + c0, H + c0 + half, 2 * H + c0, 2 * H + c0 + half};
        float t6[6];
        psumc<6, 8>(rP, MT * 16, kq, r, cols, t6);
        const float sc = rsc.get(H, p.eps);
        const float q0 = sc * t6[0], q1 = sc * t6[1], k0 = sc * t6[2], k1 = sc * t6[3], v0 = sc * t6[4], v1 = sc * t6[5];
        const unsigned qo = (unsigned)(((size_t)r * H + c0) * 4);
        stf1(rq, qo, q0 * cs - q1 * sn);
        stf1(rq, qo + half * 4, q1 * cs + q0 * sn);
        if (slot >= 0 && slot < p.cap && b == 0) {
            const unsigned o = (unsigned)((((size_t)h * p.cap + slot) * DH + i) * 2);
            st16(rK, o, f2bf(k0 * cs - k1 * sn));
            st16(rK, o + half * 2, f2bf(k1 * cs + k0 * sn));
            st16(rV, o, f2bf(v0));
            st16(rV, o + half * 2, f2bf(v1));
        }
    }
}

// merge the attention key splits, write fragments (K = H).  units: (512-column chunk, row)
template <int MT>
__device__ void step_combine(Chain &k) {
    const kp::Params &p = k.p;
    const rsrc_t ro = make_rsrc(p.o_part, p.opart_bytes), rm = make_rsrc(p.ml, p.ml_bytes);
    const rsrc_t rX = make_rsrc(p.Xf, p.xf_bytes);
    const int nch = (p.H + 511) / 512, DH = 128, ns = p.nsplit;
    for (int u = k.w * 4 + k.c; u < nch * p.rows && k.w < p.nclean; u += p.nclean * 4) {
        const int c = u % nch, r = u / nch, g = c * 64 + k.l;
        if (g >= p.H / 8) continue;
        const int h = (g * 8) / DH, d0 = (g * 8) % DH;
        const size_t base = ((size_t)r * p.n_heads + h) * ns;
        float Mx = -INFINITY;
        float ms[KOALA_NSPLIT_MAX], ls[KOALA_NSPLIT_MAX];
        f32x4 oa[KOALA_NSPLIT_MAX], oc[KOALA_NSPLIT_MAX];
#pragma unroll
        for (int s = 0; s < KOALA_NSPLIT_MAX; ++s) {
            if (s < ns) {
                const unsigned oo = (unsigned)(((base + s) * DH + d0) * 4);
                oa[s] = ldf4<AUX_SC1>(ro, oo);
                oc[s] = ldf4<AUX_SC1>(ro, oo + 16);
                ms[s] = ldf1<AUX_SC1>(rm, (unsigned)((base + s) * 8));
                ls[s] = ldf1<AUX_SC1>(rm, (unsigned)((base + s) * 8 + 4));
            } else {
                oa[s] = (f32x4){0.f, 0.f, 0.f, 0.f};
                oc[s] = (f32x4){0.f, 0.f, 0.f, 0.f};
                ms[s] = -INFINITY;
                ls[s] = 0.f;
            }
        }
#pragma unroll
        for (int s = 0; s < KOALA_NSPLIT_MAX; ++s) Mx = fmaxf(Mx, ms[s]);
        f32x4 ya = {0.f, 0.f, 0.f, 0.f}, yc = {0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
#pragma unroll
        for (int s = 0; s < KOALA_NSPLIT_MAX; ++s) {
            const float wgt = (ms[s] == -INFINITY) ? 0.f : __expf(ms[s] - Mx);
            den += wgt * ls[s];
            ya += wgt * oa[s];
            yc += wgt * oc[s];
        }
        const float inv = 1.0f / den;
        const float y[8] = {ya[0] * inv, ya[1] * inv, ya[2] * inv, ya[3] * inv,
                            yc[0] * inv, yc[1] * inv, yc[2] * inv, yc[3] * inv};
        store_frag8<MT>(rX, r, g * 8, y);
    }
}

// SiLU(gate) * up from the gate/up partial sums (column 2f = gate, 2f + 1 = up), fragments (K = F).
// units: (512 outputs, row)
template <int MT>
__device__ void step_silu(Chain &k, const Kind &kgu) {
    const kp::Params &p = k.p;
    const rsrc_t rP = make_rsrc(p.part, p.part_bytes), rS = make_rsrc(p.sums, p.sums_bytes);
    const rsrc_t rX = make_rsrc(p.Xf, p.xf_bytes);
    const int nch = (p.F / 8 + 63) / 64;
    for (int u = k.w * 4 + k.c; u < nch * p.rows && k.w < p.nclean; u += p.nclean * 4) {
        const int c = u % nch, r = u / nch, g = c * 64 + k.l;
        if (g >= p.F / 8) continue;
        const RowScale rsc(rS, (p.H + 511) / 512, p.srows, r);
        f32x4 gv[4];
        psumv<4, 2>(rP, MT * 16, kgu, r, g * 16, gv);
        float gu[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) gu[e] = gv[e >> 2][e & 3];
        const float sc = rsc.get(p.H, p.eps);
        float y[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float a = sc * gu[2 * e];
            y[e] = a / (1.0f + __expf(-a)) * (sc * gu[2 * e + 1]);
        }
        store_frag8<MT>(rX, r, g * 8, y);
    }
}

// Tree-masked attention of one (key split, head) unit by the four chain waves of a workgroup: the scheme of
// the stand-alone attention kernel (S^T = K Q^T and O^T = V^T P^T on MFMA, probabilities stay in place as the
// B operand, V transposed through a per-wave LDS tile, online softmax), for head_dim 128.
template <int MT>
__device__ void attn_unit(Chain &k, unsigned char *smem, int s, int h, rsrc_t rK, rsrc_t rV) {
    const kp::Params &p = k.p;
    constexpr int DH = 128, KS = DH / 32, DT = DH / 16, VS = DH * 2 + 8, LPR = DH / 8, VI = DH / 16;
    u32x4 *qf = (u32x4 *)smem;                                        // [MT][KS][2][64]
    unsigned char *vt_all = smem + (size_t)MT * KS * 2 * 64 * 16;     // [4 waves][32][VS]
    const int wave = k.c, l = k.l, li = l & 15, lg = l >> 4, tid = wave * 64 + l;
    unsigned char *vt = vt_all + (size_t)wave * 32 * VS;
    const float scale = rsqrtf((float)DH);
    const rsrc_t rq = make_rsrc(p.qrot, p.qrot_bytes), ro = make_rsrc(p.o_part, p.opart_bytes);
    const rsrc_t rm = make_rsrc(p.ml, p.ml_bytes);
    const int nsplit = p.nsplit, rows = p.rows, H = p.H;
    const int kv_end = min(p.meta.kv_end[0], p.cap);
    int chunk = (kv_end + nsplit - 1) / nsplit;
    chunk = (chunk + 31) / 32 * 32;
    const int j0 = s * chunk, j1 = min(kv_end, j0 + chunk);
    const int nsteps = j1 > j0 ? (j1 - j0 + 31) / 32 : 0;
    const unsigned hb = (unsigned)((size_t)h * p.cap * DH * 2);   // byte offset of this head's rows
    u32x4 kf[2][KS], vr[VI];
    auto load_step = [&](int st) {
        const int k0 = j0 + st * 32;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int key = min(k0 + 16 * j + li, p.cap - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[j][ks] = ld128<AUX_SC1>(rK, hb + (unsigned)(((size_t)key * DH + ks * 32 + 8 * lg) * 2));
        }
#pragma unroll
        for (int i = 0; i < VI; ++i) {
            const int key = min(k0 + i * (64 / LPR) + l / LPR, p.cap - 1);
            vr[i] = ld128<AUX_SC1>(rV, hb + (unsigned)(((size_t)key * DH + (l % LPR) * 8) * 2));
        }
    };
    if (wave < nsteps) load_step(wave);
    for (int u = tid; u < MT * KS * 64; u += 256) {
        const int lane = u & 63, ks = (u >> 6) % KS, mt = (u >> 6) / KS;
        const int row = mt * 16 + (lane & 15);
        float y[8];
        if (row < rows) {
            const unsigned qo = (unsigned)(((size_t)row * H + h * DH + ks * 32 + 8 * (lane >> 4)) * 4);
            const f32x4 a = ldf4<AUX_SC1>(rq, qo), b = ldf4<AUX_SC1>(rq, qo + 16);
            y[0] = a[0] * scale; y[1] = a[1] * scale; y[2] = a[2] * scale; y[3] = a[3] * scale;
            y[4] = b[0] * scale; y[5] = b[1] * scale; y[6] = b[2] * scale; y[7] = b[3] * scale;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = 0.f;
        }
        uint32_t hi[8], lo[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            hi[e] = f2bf(y[e]);
            lo[e] = f2bf(y[e] - bf2f(hi[e]));
        }
        u32x4 a, c;
        a.x = hi[0] | (hi[1] << 16); a.y = hi[2] | (hi[3] << 16); a.z = hi[4] | (hi[5] << 16); a.w = hi[6] | (hi[7] << 16);
        c.x = lo[0] | (lo[1] << 16); c.y = lo[2] | (lo[3] << 16); c.z = lo[4] | (lo[5] << 16); c.w = lo[6] | (lo[7] << 16);
        qf[((mt * KS + ks) * 2 + 0) * 64 + lane] = a;
        qf[((mt * KS + ks) * 2 + 1) * 64 + lane] = c;
    }
    int nvis[MT], base[MT];
    uint64_t mask[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int row = mt * 16 + li;
        const bool ok = row < rows;
        const int r = ok ? row : 0;
        nvis[mt] = ok ? p.meta.row_nvis[r] : 0;
        base[mt] = ok ? p.meta.row_base[r] : 0;
        mask[mt] = ok ? p.meta.row_mask[r] : 0ull;
    }
    f32x4 acc_o[MT][DT];
    float m_run[MT], l_run[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        m_run[mt] = -INFINITY;
        l_run[mt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) acc_o[mt][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    LDS_RELEASE();
    chain_sync(k);
    for (int st = wave; st < nsteps; st += 4) {
        const int k0 = j0 + st * 32;
        f32x4 sc[2][MT];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) sc[j][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const bf16x8 qh = __builtin_bit_cast(bf16x8, qf[((mt * KS + ks) * 2 + 0) * 64 + l]);
                const bf16x8 ql = __builtin_bit_cast(bf16x8, qf[((mt * KS + ks) * 2 + 1) * 64 + l]);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const bf16x8 a = __builtin_bit_cast(bf16x8, kf[j][ks]);
                    sc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qh, sc[j][mt], 0, 0, 0);
                    sc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ql, sc[j][mt], 0, 0, 0);
                }
            }
#pragma unroll
        for (int i = 0; i < VI; ++i) {
            const int kl = i * (64 / LPR) + l / LPR;
            u64_lds *dst = (u64_lds *)(vt + (size_t)kl * VS + (l % LPR) * 16);
            const bool in = k0 + kl < j1;
            dst[0] = in ? ((unsigned long long)vr[i].y << 32 | vr[i].x) : 0ull;
            dst[1] = in ? ((unsigned long long)vr[i].w << 32 | vr[i].z) : 0ull;
        }
        if (st + 4 < nsteps) load_step(st + 4);
        bf16x8 ph[MT], pl[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float pr[8];
            float tmax = -INFINITY;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = k0 + 16 * (e >> 2) + 4 * lg + (e & 3);
                const unsigned rel = (unsigned)(key - base[mt]);
                const uint32_t half = rel < 32u ? (uint32_t)mask[mt] : (uint32_t)(mask[mt] >> 32);
                const bool bit = rel < 64u && ((half >> (rel & 31u)) & 1u);
                const bool vis = key < j1 && (key < nvis[mt] || bit);
                pr[e] = vis ? sc[e >> 2][mt][e & 3] : -INFINITY;
                tmax = fmaxf(tmax, pr[e]);
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float m_new = fmaxf(m_run[mt], tmax);
            const float alpha = (m_run[mt] == -INFINITY) ? 0.f : __expf(m_run[mt] - m_new);
            float ps = 0.f;
            uint32_t hi[8], lo[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = (pr[e] == -INFINITY) ? 0.f : __expf(pr[e] - m_new);
                ps += v;
                hi[e] = f2bf(v);
                lo[e] = f2bf(v - bf2f(hi[e]));
            }
            l_run[mt] = l_run[mt] * alpha + ps;
            m_run[mt] = m_new;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                acc_o[mt][dt][0] *= alpha; acc_o[mt][dt][1] *= alpha;
                acc_o[mt][dt][2] *= alpha; acc_o[mt][dt][3] *= alpha;
            }
            u32x4 a, c;
            a.x = hi[0] | (hi[1] << 16); a.y = hi[2] | (hi[3] << 16); a.z = hi[4] | (hi[5] << 16); a.w = hi[6] | (hi[7] << 16);
            c.x = lo[0] | (lo[1] << 16); c.y = lo[2] | (lo[3] << 16); c.z = lo[4] | (lo[5] << 16); c.w = lo[6] | (lo[7] << 16);
            ph[mt] = __builtin_bit_cast(bf16x8, a);
            pl[mt] = __builtin_bit_cast(bf16x8, c);
        }
        const u16_alias *vt16 = (const u16_alias *)vt;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            uint32_t wv[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const int ka = 16 * ((2 * e2) >> 2) + 4 * lg + ((2 * e2) & 3);
                const uint32_t v0 = vt16[(size_t)ka * (VS / 2) + dt * 16 + li];
                const uint32_t v1 = vt16[(size_t)(ka + 1) * (VS / 2) + dt * 16 + li];
                wv[e2] = v0 | (v1 << 16);
            }
            u32x4 a;
            a.x = wv[0]; a.y = wv[1]; a.z = wv[2]; a.w = wv[3];
            const bf16x8 va = __builtin_bit_cast(bf16x8, a);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc_o[mt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, ph[mt], acc_o[mt][dt], 0, 0, 0);
                acc_o[mt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pl[mt], acc_o[mt][dt], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        l_run[mt] += __shfl_xor(l_run[mt], 16);
        l_run[mt] += __shfl_xor(l_run[mt], 32);
    }
    LDS_RELEASE();
    chain_sync(k);
    float *mo = (float *)smem;                         // [3 waves][MT][DT][64][4]
    float *mm = mo + (size_t)3 * MT * DT * 256;        // [3 waves][MT][64][2]
    if (wave > 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                *(f32x4 *)(mo + ((((size_t)(wave - 1) * MT + mt) * DT + dt) * 64 + l) * 4) = acc_o[mt][dt];
            mm[(((wave - 1) * MT + mt) * 64 + l) * 2 + 0] = m_run[mt];
            mm[(((wave - 1) * MT + mt) * 64 + l) * 2 + 1] = l_run[mt];
        }
    }
    LDS_RELEASE();
    chain_sync(k);
    if (wave == 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float M = m_run[mt];
#pragma unroll
            for (int w2 = 0; w2 < 3; ++w2) M = fmaxf(M, mm[((w2 * MT + mt) * 64 + l) * 2]);
            const float a0 = (m_run[mt] == -INFINITY) ? 0.f : __expf(m_run[mt] - M);
            float lsum = l_run[mt] * a0;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                acc_o[mt][dt][0] *= a0; acc_o[mt][dt][1] *= a0; acc_o[mt][dt][2] *= a0; acc_o[mt][dt][3] *= a0;
            }
#pragma unroll
            for (int w2 = 0; w2 < 3; ++w2) {
                const float mw = mm[((w2 * MT + mt) * 64 + l) * 2];
                if (mw == -INFINITY) continue;
                const float aw = __expf(mw - M);
                lsum += aw * mm[((w2 * MT + mt) * 64 + l) * 2 + 1];
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const f32x4 o = *(const f32x4 *)(mo + ((((size_t)w2 * MT + mt) * DT + dt) * 64 + l) * 4);
                    acc_o[mt][dt][0] += aw * o[0]; acc_o[mt][dt][1] += aw * o[1];
                    acc_o[mt][dt][2] += aw * o[2]; acc_o[mt][dt][3] += aw * o[3];
                }
            }
            const int row = mt * 16 + li;
            if (row < rows) {
                const size_t e = ((size_t)row * p.n_heads + h) * nsplit + s;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) stf4(ro, (unsigned)((e * DH + dt * 16 + 4 * lg) * 4), acc_o[mt][dt]);
                if (lg == 0) {
                    stf1(rm, (unsigned)(e * 8), M);
                    stf1(rm, (unsigned)(e * 8 + 4), lsum);
                }
            }
        }
    }
    LDS_RELEASE();
    chain_sync(k);   // the LDS area is free for the next unit
}

// ---------------------------------------------------------------------------------------------
// the kernel
// ---------------------------------------------------------------------------------------------
template <int MT>
__global__ __launch_bounds__(512) void k_layers_persistent(kp::Params p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    Shared &sh = *(Shared *)lds_raw;
    constexpr int XT = MT * 256;                        // 16-byte words per activation tile (64 k)
    u32x4 *xring = (u32x4 *)sh.area;                    // [XR][XT]
    f32x4 *pstage = (f32x4 *)(sh.area + XR * XT * 16);  // [4 stream waves][4 * MT * 64]
    Ctl *ctl = &sh.ctl;
    const int wave = RFL((int)(threadIdx.x >> 6)), l = threadIdx.x & 63;
    const int w = blockIdx.x, G = gridDim.x;
    for (int i = threadIdx.x; i < (int)(sizeof(Ctl) / 4); i += blockDim.x) ((int *)ctl)[i] = 0;
    for (int i = threadIdx.x; i < 4 * p.L; i += blockDim.x) {
        const kp::Layer &ly = p.layers[i >> 2];
        const int kx = i & 3;
        const unsigned long long a =
            (unsigned long long)(kx == G_QKV ? ly.wqkv : kx == G_O ? ly.wo : kx == G_GU ? ly.wgu : ly.wdown);
        sh.wtab[i][0] = (unsigned)a;
        sh.wtab[i][1] = (unsigned)(a >> 32);
        const unsigned long long b = (unsigned long long)(kx == 0 ? ly.in_norm : kx == 1 ? ly.post_norm : kx == 2 ? ly.kc : ly.vc);
        sh.ltab[i][0] = (unsigned)b;
        sh.ltab[i][1] = (unsigned)(b >> 32);
    }
    __syncthreads();
    if (threadIdx.x < 4) {
        const int g = threadIdx.x;
        const int N = g == G_QKV ? 3 * p.H : g == G_GU ? 2 * p.F : p.H, K = g == G_DOWN ? p.F : p.H;
        Kind kd;
        kd.Npad = (N + 63) / 64 * 64;
        kd.nrb = kd.Npad / 64;
        kd.KT = K / 64;
        kd.total = ((kd.nrb + 3) / 4) * kd.KT;
        kd.geff = kd.total < G ? kd.total : G;
        kd.t0 = sk_start(w, kd.total, kd.geff);
        kd.n = sk_start(w + 1, kd.total, kd.geff) - kd.t0;
        kd.pad_ = 0;
        ctl->kind[g] = kd;
    }
    __syncthreads();
    const int Mp = MT * 16, ng = 4 * p.L;

    if (wave < 4) {
        // ============================================================== stream wave
        u32x4 wr[NS][8];
        int seq = 0, nflush = 0, dead = 0;
        f32x4 acc[4][MT];
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[t][m] = (f32x4){0.f, 0.f, 0.f, 0.f};
        // tile cursors of the current projection: loads run NS tiles ahead of the products
        int n = 0, KT = 1, nrb = 0, li = 0, l_rg = 0, l_k = 0, ci = 0, c_rg = 0, c_k = 0;
        rsrc_t rs = make_rsrc(p.layers, 0);
        // always 8 loads per slot so that the waits the compiler derives are static; where there is no tile the
        // offset lies past the end of the buffer: such a load touches no memory and returns zeros
#define ISSUE(S)                                                                                         \
        {                                                                                                \
            const int rb = l_rg * 4 + wave;                                                              \
            const bool ok = li < n && rb < nrb;                                                          \
            const unsigned off = ok ? (unsigned)(((size_t)rb * KT + l_k) * 8192u) + (unsigned)l * 16u : OOB; \
            _Pragma("unroll") for (int j = 0; j < 8; ++j) wr[S][j] = ld128<AUX_NT>(rs, off + (ok ? j * 1024u : 0u)); \
            if (li < n) {                                                                                \
                ++li; ++l_k;                                                                             \
                if (l_k == KT) { l_k = 0; ++l_rg; }                                                      \
            }                                                                                            \
        }
#define FLUSH()                                                                                          \
        {                                                                                                \
            const long long tb = wall_clock64();                                                         \
            while (LDS_LD(&ctl->p_taken[wave]) != nflush) {                                              \
                __builtin_amdgcn_s_sleep(1);                                                             \
                if (LDS_LD(&ctl->abort_l) || wall_clock64() - tb > TIMEOUT_TICKS) { dead = 1; LDS_ST(&ctl->abort_l, 1); break; } \
            }                                                                                            \
            LDS_ACQUIRE();                                                                               \
            f32x4 *ps = pstage + wave * (4 * MT * 64);                                                   \
            _Pragma("unroll") for (int t = 0; t < 4; ++t)                                                \
                _Pragma("unroll") for (int m = 0; m < MT; ++m) {                                         \
                    ps[(t * MT + m) * 64 + l] = acc[t][m];                                               \
                    acc[t][m] = (f32x4){0.f, 0.f, 0.f, 0.f};                                             \
                }                                                                                        \
            LDS_RELEASE();                                                                               \
            ++nflush;                                                                                    \
            if (l == 0) LDS_ST(&ctl->p_ready[wave], nflush);                                             \
        }
#ifdef KOALA_PL_TW
#define TT(I) if (ttile) sh.tl[tli][I] = wall_clock64();
#define TT_DECL const bool ttile = p.trace && w == KOALA_PL_TW && wave == 0 && l == 0 && (gcur >> 2) == 5 && tli < 64;
#define TT_NEXT if (ttile) ++tli;
#else
#define TT(I)
#define TT_DECL
#define TT_NEXT
#endif
#define STEP(S)                                                                                          \
        if (ci < n && !dead) {                                                                           \
            const int xs = seq % XR;                                                                     \
            const long long tb = wall_clock64();                                                         \
            TT_DECL TT(0)                                                                                \
            while (LDS_LD(&ctl->xflag[xs]) != seq + 1) {                                                 \
                __builtin_amdgcn_s_sleep(1);                                                             \
                if (LDS_LD(&ctl->abort_l) || wall_clock64() - tb > TIMEOUT_TICKS) { dead = 1; LDS_ST(&ctl->abort_l, 1); break; } \
            }                                                                                            \
            LDS_ACQUIRE();                                                                               \
            TT(1)                                                                                        \
            if (!dead) {                                                                                 \
                const u32x4 *xt = xring + xs * XT;                                                       \
                if (c_rg * 4 + wave < nrb) {                                                             \
                    _Pragma("unroll") for (int s = 0; s < 2; ++s) {                                      \
                        bf16x8 xh[MT], xl[MT];                                                           \
                        _Pragma("unroll") for (int m = 0; m < MT; ++m) {                                 \
                            xh[m] = __builtin_bit_cast(bf16x8, xt[((s * MT + m) * 2 + 0) * 64 + l]);     \
                            xl[m] = __builtin_bit_cast(bf16x8, xt[((s * MT + m) * 2 + 1) * 64 + l]);     \
                        }                                                                                \
                        _Pragma("unroll") for (int t = 0; t < 4; ++t)                                    \
                            _Pragma("unroll") for (int m = 0; m < MT; ++m)                               \
                                acc[t][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wr[S][t * 2 + s]), xh[m], acc[t][m], 0, 0, 0); \
                        _Pragma("unroll") for (int t = 0; t < 4; ++t)                                    \
                            _Pragma("unroll") for (int m = 0; m < MT; ++m)                               \
                                acc[t][m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wr[S][t * 2 + s]), xl[m], acc[t][m], 0, 0, 0); \
                    }                                                                                    \
                }                                                                                        \
                ++seq;                                                                                   \
                LDS_RELEASE();                                                                           \
                if (l == 0) LDS_ST(&ctl->done[wave], seq);                                               \
                ++ci; ++c_k;                                                                             \
                TT(2)                                                                                    \
                if (c_k == KT || ci == n) { FLUSH() c_k = 0; ++c_rg; }                                   \
                TT(3) TT_NEXT                                                                            \
            }                                                                                            \
        }                                                                                                \
        ISSUE(S)
#ifdef KOALA_PL_TW
        int tli = 0, gcur = 0;
#endif
        for (int g = 0; g < ng && !dead; ++g) {
            const int kx = g & 3;
#ifdef KOALA_PL_TW
            gcur = g;
#endif
            n = LDS_LD(&ctl->kind[kx].n);
            if (n == 0) continue;
            const int t0 = LDS_LD(&ctl->kind[kx].t0);
            KT = LDS_LD(&ctl->kind[kx].KT);
            nrb = LDS_LD(&ctl->kind[kx].nrb);
            li = 0; ci = 0;
            l_rg = c_rg = t0 / KT;
            l_k = c_k = t0 % KT;
            {
                const unsigned a_lo = (unsigned)LDS_LD((int *)&sh.wtab[g][0]);
                const unsigned a_hi = (unsigned)LDS_LD((int *)&sh.wtab[g][1]);
                const void *wp = (const void *)(((unsigned long long)a_hi << 32) | (unsigned long long)a_lo);
                rs = make_rsrc(wp, (unsigned)nrb * 64u * (unsigned)KT * 64u * 2u);
            }
            // the chain waves say when this projection's first loads may enter the CU's memory pipeline
            {
                const long long tb = wall_clock64();
                while (LDS_LD(&ctl->go) <= g) {
                    __builtin_amdgcn_s_sleep(1);
                    if (LDS_LD(&ctl->abort_l) || wall_clock64() - tb > TIMEOUT_TICKS) { dead = 1; LDS_ST(&ctl->abort_l, 1); break; }
                }
            }
            if (dead) break;
            ISSUE(0)
            ISSUE(1)
            ISSUE(2)
#if KOALA_PL_NS > 3
            ISSUE(3)
#endif
#if KOALA_PL_NS > 4
            ISSUE(4)
#endif
#if KOALA_PL_NS > 5
            ISSUE(5)
#endif
            while (ci < n && !dead) {
                STEP(0)
                STEP(1)
                STEP(2)
#if KOALA_PL_NS > 3
                STEP(3)
#endif
#if KOALA_PL_NS > 4
                STEP(4)
#endif
#if KOALA_PL_NS > 5
                STEP(5)
#endif
            }
        }
#ifdef KOALA_PL_TW
        if (p.trace && w == KOALA_PL_TW && wave == 0 && l == 0) {
            long long *tx = p.trace + 3 * (2 + 10 * p.L);
            tx[0] = tli;
            for (int i = 0; i < tli; ++i)
                for (int j = 0; j < 4; ++j) tx[1 + 4 * i + j] = sh.tl[i][j];
        }
#endif
    } else {
        // ============================================================== chain wave
        Chain k{p};
        k.ctl = ctl; k.c = wave - 4; k.l = l; k.w = w; k.G = G;
        k.gen = p.bar_base; k.shard_target = p.shard_base; k.cgen = 0; k.dead = false;
        // workgroups that take no part in the small steps may fetch the first projection's weights at once
        if (k.c == 0 && l == 0 && w >= p.pf_from) LDS_ST(&ctl->go, 1);
        const int c = k.c;
        int seq_base = 0;
        const rsrc_t rX = make_rsrc(p.Xf, p.xf_bytes), rP = make_rsrc(p.part, p.part_bytes);
        Kind kd[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            kd[g].nrb = LDS_LD(&ctl->kind[g].nrb); kd[g].KT = LDS_LD(&ctl->kind[g].KT);
            kd[g].total = LDS_LD(&ctl->kind[g].total); kd[g].geff = LDS_LD(&ctl->kind[g].geff);
            kd[g].Npad = LDS_LD(&ctl->kind[g].Npad); kd[g].t0 = LDS_LD(&ctl->kind[g].t0);
            kd[g].n = LDS_LD(&ctl->kind[g].n); kd[g].pad_ = 0;
        }
        // one GEMM phase: feed this workgroup's activation tiles to the ring, write its partial sums out
        // one GEMM phase: every chain wave feeds every fourth activation tile of this workgroup to the ring (requested
        // before its ring slot is free) and writes out the partial sums of the stream wave with its number
        int ndrained = 0;
        auto gemm_phase = [&](const Kind &d, int g) {
            const int t0 = d.t0, n = d.n;
            if (c == 0 && l == 0 && w < p.pf_from) LDS_ST(&ctl->go, g + 1);
            if (n > 0) {
                const int rg0 = t0 / d.KT, rg1 = (t0 + n - 1) / d.KT;
                int feed = c, drg = rg0;
                long long tb = wall_clock64();
                u32x4 v[MT * 4];
                bool loaded = false;
                while ((feed < n || drg <= rg1) && !k.dead) {
                    bool progressed = false;
                    if (feed < n && !loaded) {
                        const int kt = (t0 + feed) % d.KT;
#pragma unroll
                        for (int u = 0; u < MT * 4; ++u)
                            v[u] = ld128<AUX_X>(rX, (unsigned)(((size_t)kt * XT + u * 64 + l) * 16));
                        loaded = true;
                    }
                    if (feed < n) {
                        const int seq = seq_base + feed;
                        int md = LDS_LD(&ctl->done[0]);
                        md = min(md, LDS_LD(&ctl->done[1]));
                        md = min(md, LDS_LD(&ctl->done[2]));
                        md = min(md, LDS_LD(&ctl->done[3]));
                        if (seq < XR || md >= seq - XR + 1) {
                            LDS_ACQUIRE();
                            u32x4 *dst = xring + (seq % XR) * XT;
#pragma unroll
                            for (int u = 0; u < MT * 4; ++u) dst[u * 64 + l] = v[u];
                            LDS_RELEASE();
                            if (l == 0) LDS_ST(&ctl->xflag[seq % XR], seq + 1);
                            feed += 4;
                            loaded = false;
                            progressed = true;
                        }
                    }
                    if (drg <= rg1 && LDS_LD(&ctl->p_ready[c]) > ndrained) {
                        LDS_ACQUIRE();
                        const int rb = drg * 4 + c;
                        if (rb < d.nrb) {
                            const int sl = w - sk_owner(drg * d.KT, d.total, d.geff);
                            const f32x4 *ps = pstage + c * (4 * MT * 64);
                            const int li = l & 15, lgp = l >> 4;
                            const size_t sbase = (size_t)sl * Mp * d.Npad;
#pragma unroll
                            for (int t = 0; t < 4; ++t)
#pragma unroll
                                for (int m = 0; m < MT; ++m) {
                                    const f32x4 val = ps[(t * MT + m) * 64 + l];
                                    const int row = m * 16 + li, nn = rb * 64 + 16 * t + 4 * lgp;
                                    stf4(rP, (unsigned)((sbase + (size_t)row * d.Npad + nn) * 4), val);
                                }
                        }
                        LDS_RELEASE();
                        ++ndrained;
                        if (l == 0) LDS_ST(&ctl->p_taken[c], ndrained);
                        ++drg;
                        progressed = true;
                    }
                    if (!progressed) {
                        __builtin_amdgcn_s_sleep(1);
                        if (LDS_LD(&ctl->abort_l) || wall_clock64() - tb > TIMEOUT_TICKS) { LDS_ST(&ctl->abort_l, 1); k.dead = true; }
                    } else {
                        tb = wall_clock64();
                    }
                }
                seq_base += n;
            }
            // the arrival goes first, then the next projection's first weight tiles (they overlap the small step
            // that follows)
            grid_barrier(k, true, (w >= p.pf_from && g + 1 < 4 * p.L) ? g + 2 : 0);
        };
        if (p.trace && w == 0 && c == 0 && l == 0) p.trace[0] = wall_clock64();
        for (int ly = 0; ly < p.L && !k.dead; ++ly) {
            const void *lp[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned a_lo = (unsigned)LDS_LD((int *)&sh.ltab[4 * ly + i][0]);
                const unsigned a_hi = (unsigned)LDS_LD((int *)&sh.ltab[4 * ly + i][1]);
                lp[i] = (const void *)(((unsigned long long)a_hi << 32) | (unsigned long long)a_lo);
            }
            const rsrc_t rK = make_rsrc(lp[2], p.kv_layer_bytes), rV = make_rsrc(lp[3], p.kv_layer_bytes);
            step_fold<MT>(k, ly == 0 ? 0 : 1, kd[G_DOWN], lp[0], true);
            grid_barrier(k, false, 0);
            gemm_phase(kd[G_QKV], 4 * ly + G_QKV);
            if (k.dead) break;
            step_rope<MT>(k, kd[G_QKV], rK, rV);
            grid_barrier(k, false, 0);
            if (k.dead) break;
            for (int u = w; u < p.nsplit * p.n_heads; u += G) attn_unit<MT>(k, sh.area, u % p.nsplit, u / p.nsplit, rK, rV);
            grid_barrier(k, true, 0);
            if (k.dead) break;
            step_combine<MT>(k);
            grid_barrier(k, false, 0);
            gemm_phase(kd[G_O], 4 * ly + G_O);
            if (k.dead) break;
            step_fold<MT>(k, 1, kd[G_O], lp[1], true);
            grid_barrier(k, false, 0);
            gemm_phase(kd[G_GU], 4 * ly + G_GU);
            if (k.dead) break;
            step_silu<MT>(k, kd[G_GU]);
            grid_barrier(k, false, 0);
            gemm_phase(kd[G_DOWN], 4 * ly + G_DOWN);
        }
        if (!k.dead) step_fold<MT>(k, 1, kd[G_DOWN], nullptr, false);   // the last down projection into x
        __builtin_amdgcn_s_waitcnt(0x0F70);
        if (p.trace && w == 0 && c == 0 && l == 0) p.trace[1 + 10 * p.L] = wall_clock64();
        if (k.dead && l == 0 && c == 0 && p.abort_host) *p.abort_host = 1;
    }
}

}  // namespace

namespace kp {

bool supported(int rows, int batch, int head_dim, int n_layers) {
    return batch == 1 && rows >= 1 && rows <= 32 && head_dim == 128 && n_layers <= MAX_LAYERS;
}

// slots the partial-sum buffer needs for the stream-K cut with G workgroups, in floats per 16 rows
size_t part_floats_per_row(int H, int F, int G) {
    size_t worst = 0;
    const int NK[4][2] = {{3 * H, H}, {H, H}, {2 * F, H}, {H, F}};
    for (auto &nk : NK) {
        const int Npad = (nk[0] + 63) / 64 * 64, KT = nk[1] / 64, total = ((Npad / 64 + 3) / 4) * KT;
        const int geff = total < G ? total : G, q = total / geff;
        const int slots = (KT - 1 + q - 1) / q + 1;
        worst = std::max(worst, (size_t)slots * Npad);
    }
    return worst;
}

hipError_t launch(hipStream_t st, const Params &p, int MT, int G) {
    // the stream-K cut is computed in 32-bit arithmetic: (tiles of the largest projection + 1) * G must fit
    const unsigned long long NK[4][2] = {{3ull * p.H, (unsigned long long)p.H}, {(unsigned long long)p.H, (unsigned long long)p.H},
                                         {2ull * p.F, (unsigned long long)p.H}, {(unsigned long long)p.H, (unsigned long long)p.F}};
    unsigned long long tiles = 0;
    for (auto &nk : NK) tiles = std::max(tiles, ((nk[0] + 255) / 256) * (nk[1] / 64));
    if ((tiles + 1) * (unsigned long long)G >= 0xFFFFFFFFull || p.H % 64 || p.F % 64 || p.L > MAX_LAYERS)
        return hipErrorInvalidValue;
    Params q = p;
    void *args[] = {&q};
    const void *fn = MT == 1 ? (const void *)k_layers_persistent<1> : (const void *)k_layers_persistent<2>;
    static bool attr_done[2] = {false, false};
    if (!attr_done[MT - 1]) {
        const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(Shared));
        if (e != hipSuccess) return e;
        attr_done[MT - 1] = true;
    }
    return hipLaunchCooperativeKernel(fn, dim3(G), dim3(512), args, sizeof(Shared), st);
}

}  // namespace kp
