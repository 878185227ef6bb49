// bf16 weight-streaming path for gfx950.
//
// Every projection of the draft-then-verify iteration has only a handful of activation rows
// (the tree nodes) against a large weight matrix, so it is bound by how fast the weights
// stream out of HBM.  The kernels here are built around that:
//   * weights are stored fragment-major (see koala.h) as fp16 images of their bf16 values (exact: eight
//     significant bits fit eleven; k_weights_to_f16 below converts a packed matrix once): one wave load
//     instruction reads 1 KiB of contiguous memory and lands exactly in the A operand of a 16x16x32 fp16 MFMA;
//   * GEMM inputs are written by their producers as fp16 in MFMA fragment order (eleven significant bits
//     against the eight of a bf16 activation; products are exact and accumulate in fp32); RMSNorm is split
//     into the gain (applied by the producer) and the row scale (applied by whoever consumes the GEMM
//     result), since the GEMM is linear in the row scale;
//   * K is split over workgroups; partial sums go to a scratch buffer that the consumer
//     kernel adds up in a fixed order (deterministic, no float atomics).
#include "koala_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
struct __attribute__((may_alias, aligned(8))) u64_pair { uint32_t x, y; };
struct __attribute__((may_alias, aligned(8))) f32_pair { float x, y; };

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }
// (a, b) as bfloat16 pairs hi and lo with a ~ hi.x + lo.x, b ~ hi.y + lo.y (~16 mantissa bits): one packed
// round-to-nearest-even conversion per pair
struct HiLo { uint32_t hi, lo; };
__device__ __forceinline__ HiLo split_pair(float a, float b) {
    HiLo r;
    r.hi = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){a, b}, bf16x2));
    r.lo = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){a - __uint_as_float(r.hi << 16),
                                                                          b - __uint_as_float(r.hi & 0xFFFF0000u)}, bf16x2));
    return r;
}
// first of the n units that split i of S takes (units are dealt out as evenly as whole numbers allow).  In 32-bit
// unsigned arithmetic on purpose: i * n stays far below 2^32 here, and a 64-bit division is a long instruction
// sequence in front of a kernel's first load.
__device__ __forceinline__ int split_begin(int i, int n, int S) {
    return S == 1 ? i * n : (int)((unsigned)(i * n) / (unsigned)S);
}
// (a, b) as a pair of fp16 (round to nearest even), values beyond the fp16 range clamped to its largest finite one
__device__ __forceinline__ uint32_t half_pair(float a, float b) {
    a = __builtin_fminf(__builtin_fmaxf(a, -65504.f), 65504.f);
    b = __builtin_fminf(__builtin_fmaxf(b, -65504.f), 65504.f);
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){a, b}, f16x2));
}
// eight values -> the 16 bytes of a GEMM input fragment lane
__device__ __forceinline__ u32x4 half8(const float *y) {
    return (u32x4){half_pair(y[0], y[1]), half_pair(y[2], y[3]), half_pair(y[4], y[5]), half_pair(y[6], y[7])};
}
// eight values -> the hi and lo 16-byte pieces of a fragment lane (bf16 pairs: the attention kernel's operands)
__device__ __forceinline__ void split8(const float *y, u32x4 &h, u32x4 &w) {
    const HiLo p0 = split_pair(y[0], y[1]), p1 = split_pair(y[2], y[3]), p2 = split_pair(y[4], y[5]), p3 = split_pair(y[6], y[7]);
    h = (u32x4){p0.hi, p1.hi, p2.hi, p3.hi};
    w = (u32x4){p0.lo, p1.lo, p2.lo, p3.lo};
}
__device__ __forceinline__ uint32_t f2bf(float v) {  // round to nearest even
    uint32_t u = __float_as_uint(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// ---------------------------------------------------------------------------------------------
// Packed GEMM.  Wp: [Npad/64][K/64] tiles of 64 rows x 64 k, each tile = 8 fragments
// (t = row/16, s = k/32) of 64 lanes x 16 B; lane = (row%16) + 16*((k%32)/8).
// Xf: [K/32][MTT][64 lanes] x 16 B (fp16); lane = (m%16) + 16*((k%32)/8); a launch handles the MT
//     activation tiles mt0 .. mt0+MT-1 of the MTT present.
// P:  [S][MTT*16][Npad] fp32 partial sums; split sp covers 128-k chunks [sp*nch/S, (sp+1)*nch/S).
// Workgroup = 4 waves; wave w owns row block wb*4 + w (64 rows); the X chunk is shared in LDS.
// ---------------------------------------------------------------------------------------------
template <int MT, int RS>
__global__ __launch_bounds__(256 * RS, RS > 1 ? 1 : MT == 4 ? 2 : 3) void k_gemm_packed(
    const u32x4 *__restrict__ Wp, const u32x4 *__restrict__ Xf, float *__restrict__ P, int Npad, int K, int S, int nwb,
    int MTT, int mt0) {
    // RS waves share each 64-row weight block and split the activation tiles between them (wave w of 4 * RS:
    // row block w % 4, tiles (w / 4) * MT ..): one pass over the weights then serves MT * RS tiles.  The waves
    // that share a block load the same fragments at about the same time, so HBM sees them once.
    extern __shared__ u32x4 xs[];            // [2][XCH]
    constexpr int MTW = MT * RS;             // activation tiles of the workgroup
    constexpr int NT = 256 * RS;
    constexpr int XCH = 4 * MTW * 64;        // 16-byte units of X per 128-k chunk
    constexpr int XPT = XCH / NT;            // per thread
    const int wave = threadIdx.x >> 6, l = threadIdx.x & 63, li = l & 15, lg = l >> 4;
    const int wv = wave & 3, rs = wave >> 2;
    const int wb = blockIdx.x % nwb, sp = blockIdx.x / nwb;
    const int nch = K / 128;
    const int c_begin = split_begin(sp, nch, S), c_end = split_begin(sp + 1, nch, S);
    const int nchunks = c_end - c_begin;
    const int rb = wb * 4 + wv;
    const bool active = rb < Npad / 64;
    const u32x4 *wsrc = Wp + ((size_t)(active ? rb : 0) * (K / 64) + (size_t)c_begin * 2) * 512 + l;
    // 16-byte unit u of chunk c lives at xsrc + (c*4 + u / (MTW*64)) * MTT*64 + u % (MTW*64)
    const u32x4 *xsrc = Xf + (size_t)c_begin * 4 * MTT * 64 + (size_t)mt0 * 64;
    auto xaddr = [&](int c, int u) { return xsrc + ((size_t)c * 4 + u / (MTW * 64)) * (MTT * 64) + u % (MTW * 64); };
    f32x4 acc[4][MT];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[t][m] = (f32x4){0.f, 0.f, 0.f, 0.f};
    u32x4 wr[2][8];
    u32x4 xr[XPT];
    const int nb = nchunks * 2;
    auto wload = [&](int b, int slot) {
#pragma unroll
        for (int j = 0; j < 8; ++j)   // RS > 1: cacheable, so that the second wave of a row block finds the tile in L2
            wr[slot][j] = RS > 1 ? wsrc[(size_t)b * 512 + j * 64] : __builtin_nontemporal_load(wsrc + (size_t)b * 512 + j * 64);
    };
    if (nchunks > 0) {
        // X loads first, weight loads right behind them: the wait for X then leaves the weight loads in flight
#pragma unroll
        for (int i = 0; i < XPT; ++i) xr[i] = *xaddr(0, threadIdx.x + NT * i);
        if (active) {
            wload(0, 0);
            wload(1, 1);
        }
#pragma unroll
        for (int i = 0; i < XPT; ++i) xs[threadIdx.x + NT * i] = xr[i];
    }
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const bool more = c + 1 < nchunks;
        if (more) {
#pragma unroll
            for (int i = 0; i < XPT; ++i) xr[i] = *xaddr(c + 1, threadIdx.x + NT * i);
        }
        const u32x4 *xc = xs + (c & 1) * XCH;
        if (active) {
#pragma unroll
            for (int bb = 0; bb < 2; ++bb) {
                f16x8 a[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) a[j] = __builtin_bit_cast(f16x8, wr[bb][j]);
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const u32x4 *xk = xc + (bb * 2 + s) * (MTW * 64) + rs * (MT * 64);
                    f16x8 xv[MT];
#pragma unroll
                    for (int m = 0; m < MT; ++m) xv[m] = __builtin_bit_cast(f16x8, xk[m * 64 + l]);
#pragma unroll
                    for (int t = 0; t < 4; ++t)
#pragma unroll
                        for (int m = 0; m < MT; ++m)
                            acc[t][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[t * 2 + s], xv[m], acc[t][m], 0, 0, 0);
                }
                // reloading a batch only after its MFMAs keeps the register count low enough for three (MT <= 2)
                // or two (MT = 4) workgroups per CU; the other batch is in flight meanwhile
                if (2 * c + bb + 2 < nb) wload(2 * c + bb + 2, bb);
            }
        }
        if (more) {
            u32x4 *xn = xs + ((c + 1) & 1) * XCH;
#pragma unroll
            for (int i = 0; i < XPT; ++i) xn[threadIdx.x + NT * i] = xr[i];
        }
        __syncthreads();
    }
    if (active) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const int row = (mt0 + rs * MT + m) * 16 + li, n = rb * 64 + 16 * t + 4 * lg;
                *(f32x4 *)(P + ((size_t)sp * (MTT * 16) + row) * Npad + n) = acc[t][m];
            }
    }
}

// ---------------------------------------------------------------------------------------------
// Row-group GEMM with a fused epilogue.  One workgroup owns U consecutive 16-row groups of the weights
// (16 U output columns) over a K range; its waves take the 64-k tiles of that range in turn (wave w:
// tiles w, w + KW, ...) and every wave loads both operands of its tiles straight into MFMA registers -
// the U 2 KiB weight pieces and the matching activation fragments - so the streaming loop has no
// barrier and no LDS traffic.  The waves' accumulators meet at the end, in LDS, and are added in a fixed order
// (deterministic).  With S = 1 the workgroup then holds finished outputs and applies the consumer's
// element-wise step itself:
//   EPI_PARTIAL  store fp32 partial sums P[sp][row][n] (split-K, S >= 1), folded by a later kernel;
//   EPI_QKV      row scale of the pending RMSNorm, rotary embedding, queries (times 1/sqrt(head_dim)) as hi/lo
//                MFMA fragments for the attention kernel, rotated keys and values to their cache slots (bf16).  W_q / W_k rows are stored pair-interleaved
//                (koala.h), so the two halves of a rotary pair are neighbours in one lane;
//   EPI_SWIGLU   row scale, SiLU(gate) * up (rows interleaved gate, up), written as fragments of the
//                down projection's input.
// Every compute unit can take in only so many bytes per second (about 53 GB/s measured, weights and
// activations together), and with S = 1 every workgroup reads all activation fragments; U is therefore
// chosen so that one launch is one workgroup per compute unit with equal shares of the weights.
// RS > 1: RS waves share a tile position and split the MT * RS activation tiles between them.
// ---------------------------------------------------------------------------------------------
enum { EPI_PARTIAL = 0, EPI_QKV = 1, EPI_SWIGLU = 2 };

// whether the wave accumulators of k_gemm_rows are combined in halving rounds (they do not all fit in LDS at once)
constexpr bool gemm_rows_tree(int U, int MT, int NW) { return NW * U * MT > 96; }

struct GemmEpi {
    float *P;           // EPI_PARTIAL
    const float *sums;  // EPI_QKV, EPI_SWIGLU: per-chunk sums of squares of the input rows (nullptr: scale 1)
    int nparts, srows, Kn;
    float eps;
    int rows;           // valid activation rows
    RowMeta meta;       // EPI_QKV
    uint32_t *qf;       // query fragments [batch][n_heads][MTQ][DH/32][hi, lo][64 lanes][4], scaled by qscale
    bf16_t *kc, *vc;
    int H, n_heads, DH, cap, rows_per_seq, MTQ;
    float qscale;
    uint32_t *Xo;       // EPI_SWIGLU: output fragments, F = out features / 2
    int F;
};

template <int U, int MT, int RS, int NW, int PF, int EPI>
__global__ __launch_bounds__(64 * NW) void k_gemm_rows(const u32x4 *__restrict__ Wp, const u32x4 *__restrict__ Xf,
                                                       int Npad, int K, int S, GemmEpi e) {
    constexpr int MTT = MT * RS, KW = NW / RS;
    constexpr bool TREE = gemm_rows_tree(U, MT, NW);
    constexpr int NRED = TREE ? NW / 2 : NW;
    extern __shared__ __attribute__((aligned(16))) unsigned char gsm[];
    f32x4 *red = (f32x4 *)gsm;                                     // [NRED][U][MT][64]
    float *cs = (float *)(gsm + (size_t)NRED * U * MT * 64 * 16);    // EPI_QKV: [MTT*16][U][8][cos, sin]
    const int wave = threadIdx.x >> 6, l = threadIdx.x & 63, li = l & 15, lg = l >> 4;
    const int kw = wave / RS, mh = wave % RS;
    const int nunits = Npad / 16, nwg = (nunits + U - 1) / U;
    const int g = blockIdx.x % nwg, sp = blockIdx.x / nwg, ug0 = g * U;
    const int nkt = K / 64;
    const int kt0 = split_begin(sp, nkt, S), kt1 = split_begin(sp + 1, nkt, S);
    const u32x4 *w[U];   // unit j, tile kt, half s: w[j] + kt * 512 + s * 64 (a ragged last group re-reads its last unit)
#pragma unroll
    for (int j = 0; j < U; ++j) {
        const int ug = min(ug0 + j, nunits - 1);
        w[j] = Wp + ((size_t)(ug >> 2) * nkt * 8 + (ug & 3) * 2) * 64 + l;
    }
    const u32x4 *x = Xf + (size_t)mh * MT * 64 + l;

    u32x4 wr[PF][U][2], xr[PF][2][MT];
    auto load = [&](int kt, int slot) {
#pragma unroll
        for (int j = 0; j < U; ++j)
#pragma unroll
            for (int s = 0; s < 2; ++s) wr[slot][j][s] = __builtin_nontemporal_load(w[j] + (size_t)kt * 512 + s * 64);
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int m = 0; m < MT; ++m) xr[slot][s][m] = x[(size_t)(2 * kt + s) * (MTT * 64) + m * 64];
    };
    int kt = kt0 + kw;
#pragma unroll
    for (int p = 0; p < PF; ++p)
        if (kt + p * KW < kt1) load(kt + p * KW, p);

    // per-lane row data of the epilogue, fetched while the first tiles are in flight
    float rsc[MTT];
    int rslot[MTT], rbat[MTT];
    if (EPI != EPI_PARTIAL) {
#pragma unroll
        for (int m = 0; m < MTT; ++m) {
            const int row = m * 16 + li;
            const bool ok = row < e.rows;
            float tot = 0.f;
            if (e.sums && ok)
                for (int c = 0; c < e.nparts; ++c) tot += e.sums[(size_t)c * e.srows + row];
            rsc[m] = e.sums ? 1.0f / sqrtf(tot / (float)e.Kn + e.eps) : 1.f;
            if (EPI == EPI_QKV) {
                rslot[m] = ok ? e.meta.row_slot[row] : 0;
                rbat[m] = ok ? e.meta.row_b[row] : 0;
            }
        }
    }
    if (EPI == EPI_QKV) {
        const int half = e.DH / 2;
        for (int u = threadIdx.x; u < MTT * 16 * U * 8; u += 64 * NW) {
            const int dd = u & 7, j = (u >> 3) % U, row = (u >> 3) / U;
            const int n = min(ug0 + j, nunits - 1) * 16;
            const bool ok = row < e.rows && n < 2 * e.H;
            const int ddg = ((n % e.H) % e.DH) / 2 + dd;
            cs[2 * u] = ok ? e.meta.rope_cos[(size_t)row * half + ddg] : 1.f;
            cs[2 * u + 1] = ok ? e.meta.rope_sin[(size_t)row * half + ddg] : 0.f;
        }
    }

    f32x4 acc[U][MT];
#pragma unroll
    for (int j = 0; j < U; ++j)
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[j][m] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (; kt < kt1; kt += PF * KW) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            if (kt + p * KW < kt1) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
#pragma unroll
                    for (int j = 0; j < U; ++j) {
                        const f16x8 a = __builtin_bit_cast(f16x8, wr[p][j][s]);
#pragma unroll
                        for (int m = 0; m < MT; ++m)
                            acc[j][m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(
                                a, __builtin_bit_cast(f16x8, xr[p][s][m]), acc[j][m], 0, 0, 0);
                    }
                }
                if (kt + (p + PF) * KW < kt1) load(kt + (p + PF) * KW, p);
            }
        }
    }
    // The waves' sums meet in LDS.  Where it fits (TREE false) every wave stores its accumulators and the epilogue
    // adds the KW copies of a piece in wave order; otherwise the number of live accumulators is halved per round
    // (waves [n/2, n) hand theirs to waves [0, n/2)) and waves 0 .. RS-1 store the totals.  Either order is fixed,
    // so results are bit-for-bit repeatable.
    if (!TREE) {
#pragma unroll
        for (int j = 0; j < U; ++j)
#pragma unroll
            for (int m = 0; m < MT; ++m) red[((size_t)(wave * U + j) * MT + m) * 64 + l] = acc[j][m];
    } else {
#pragma unroll
        for (int n = NW; n > RS; n >>= 1) {
            const int hn = n >> 1;
            if (n < NW) __syncthreads();
            if (wave >= hn && wave < n) {
#pragma unroll
                for (int j = 0; j < U; ++j)
#pragma unroll
                    for (int m = 0; m < MT; ++m) red[((size_t)((wave - hn) * U + j) * MT + m) * 64 + l] = acc[j][m];
            }
            __syncthreads();
            if (wave < hn) {
#pragma unroll
                for (int j = 0; j < U; ++j)
#pragma unroll
                    for (int m = 0; m < MT; ++m) acc[j][m] += red[((size_t)(wave * U + j) * MT + m) * 64 + l];
            }
        }
        __syncthreads();
        if (wave < RS) {
#pragma unroll
            for (int j = 0; j < U; ++j)
#pragma unroll
                for (int m = 0; m < MT; ++m) red[((size_t)(wave * U + j) * MT + m) * 64 + l] = acc[j][m];
        }
    }
    __syncthreads();

    // output piece (j, mtt): weight rows of unit j x activation tile mtt; lane (li, lg) holds columns
    // n .. n + 3 of activation row mtt * 16 + li
    for (int u = wave; u < U * MTT; u += NW) {
        const int j = u / MTT, mtt = u % MTT, umh = mtt / MT, um = mtt % MT;
        if (ug0 + j >= nunits) continue;
        f32x4 v = red[((size_t)(umh * U + j) * MT + um) * 64 + l];
        if (!TREE) {
#pragma unroll
            for (int q = 1; q < KW; ++q) v += red[((size_t)((q * RS + umh) * U + j) * MT + um) * 64 + l];
        }
        const int row = mtt * 16 + li, n = (ug0 + j) * 16 + 4 * lg;
        if (EPI == EPI_PARTIAL) {
            *(f32x4 *)(e.P + ((size_t)sp * (MTT * 16) + row) * Npad + n) = v;
            continue;
        }
        if (row >= e.rows) continue;
        float sc = 1.f;
        int slot = 0, bat = 0;
#pragma unroll
        for (int m = 0; m < MTT; ++m)   // static indexing keeps the per-row data in registers
            if (m == mtt) { sc = rsc[m]; if (EPI == EPI_QKV) { slot = rslot[m]; bat = rbat[m]; } }
        v *= sc;
        if (EPI == EPI_QKV) {
            const int which = n / e.H, nn = n % e.H, h = nn / e.DH, r = nn % e.DH, half = e.DH / 2;
            const size_t o = (((size_t)bat * e.n_heads + h) * e.cap + slot) * e.DH;
            if (which == 2) {
                const uint32_t lo = f2bf(v[0]) | (f2bf(v[1]) << 16), hi = f2bf(v[2]) | (f2bf(v[3]) << 16);
                *(u64_pair *)(e.vc + o + r) = u64_pair{lo, hi};
            } else {
                const int dd = r >> 1;
                const float *t = cs + 2 * (((size_t)row * U + j) * 8 + 2 * lg);
                const float c0 = t[0], s0 = t[1], c1 = t[2], s1 = t[3];
                const float a0 = v[0] * c0 - v[1] * s0, b0 = v[1] * c0 + v[0] * s0;
                const float a1 = v[2] * c1 - v[3] * s1, b1 = v[3] * c1 + v[2] * s1;
                if (which == 0) {
                    // dimensions dd, dd + 1 and dd + half, dd + half + 1 of row i of its sequence
                    const int i = row - bat * e.rows_per_seq;
                    uint32_t *qt = e.qf + ((((size_t)bat * e.n_heads + h) * e.MTQ + (i >> 4)) * (e.DH / 32)) * 2 * 64 * 4;
                    const float y[4] = {a0 * e.qscale, a1 * e.qscale, b0 * e.qscale, b1 * e.qscale};
#pragma unroll
                    for (int z = 0; z < 2; ++z) {
                        const int d = dd + z * half;
                        const HiLo pr = split_pair(y[2 * z], y[2 * z + 1]);
                        const uint32_t hi = pr.hi, lo = pr.lo;
                        uint32_t *dst = qt + (((size_t)(d >> 5) * 2) * 64 + (i & 15) + 16 * ((d & 31) >> 3)) * 4 + ((d & 7) >> 1);
                        dst[0] = hi;
                        dst[64 * 4] = lo;
                    }
                } else {
                    *(uint32_t *)(e.kc + o + dd) = f2bf(a0) | (f2bf(a1) << 16);
                    *(uint32_t *)(e.kc + o + half + dd) = f2bf(b0) | (f2bf(b1) << 16);
                }
            }
        } else {   // EPI_SWIGLU
            const int f0 = n >> 1;
            if (f0 >= e.F) continue;
            const float g0 = v[0], g1 = v[2];
            const float y0 = g0 / (1.0f + __expf(-g0)) * v[1], y1 = g1 / (1.0f + __expf(-g1)) * v[3];
            const int ks = f0 >> 5, lane = li + 16 * ((f0 & 31) >> 3);
            e.Xo[(((size_t)ks * MTT + mtt) * 64 + lane) * 4 + ((f0 & 7) >> 1)] = half_pair(y0, y1);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// GEMM for many activation rows (batched verification: hundreds of rows), where the matrix pipe and the
// operand traffic, not the weight stream alone, set the pace.  One workgroup of four waves per compute unit
// (one wave per SIMD, so a wave may use the whole register file) owns 4 U weight row groups of 16 rows and up
// to MTW activation tiles over a K range.  Wave w keeps its U groups' weight fragments of the current and the
// next 64-k tile in registers (loaded straight from HBM) and all U x MTW accumulator tiles; the activation
// fragments of a 64-k tile are shared by the four waves through LDS, filled by loads that go from global
// memory to LDS directly (no staging registers), double-buffered.  Every activation fragment fetched from
// LDS feeds U MFMAs (hi) + U (lo).  Output: fp32 partial sums P[sp][row][n] like the other GEMMs.
// grid: (row-group blocks) x (activation tile blocks) x S.
// ---------------------------------------------------------------------------------------------
// acc += A * B on the matrix pipe with the accumulator tile held in place in the accumulation registers.  Written
// as an instruction of its own because the compiler's MFMA builtin, once a wave uses more than 256 registers,
// gives every result a new register and copies it back, which costs more than the MFMA itself.  An MFMA may
// follow another that wrote its accumulator operand without waiting when both name the same registers, as here.
// The compiler does not know that this is a matrix instruction and keeps none of the distances the hardware wants
// around one: `a` and `b` must not come straight out of a vector-unit instruction (loads are fine: the wait for
// their data is distance enough; a value computed in the vector unit needs a few idle cycles before the matrix
// instruction reads it, or the instruction now and then sees the register's old contents), and the result may be
// read only after mfma_settle.
__device__ __forceinline__ void mfma_acc(f32x4 &acc, f16x8 a, f16x8 b) {
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// Results of the matrix pipe may be read by other instructions only some cycles after the MFMA was issued; for
// the compiler's own MFMAs the compiler sees to that, for mfma_acc it cannot.  These statements wait (WAIT) and
// hand the accumulator tiles through, so that whatever reads them afterwards, wherever the compiler places it,
// depends on a statement that comes after the wait.
template <bool WAIT>
__device__ __forceinline__ void mfma_settle(f32x4 &a, f32x4 &b, f32x4 &c, f32x4 &d) {
    if (WAIT) asm volatile("s_nop 15\n\ts_nop 7" : "+a"(a), "+a"(b), "+a"(c), "+a"(d));
    else asm volatile("" : "+a"(a), "+a"(b), "+a"(c), "+a"(d));
}

// 16 bytes per lane from LDS at base + a constant byte offset (below 64 KiB), as an instruction of its own: the
// result may be used only after a wait that covers it (wait_lds_reads).
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
__device__ __forceinline__ u32x4 lds_read16(lds_u32x4 *base, int byte_offset) {
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(base), "n"(byte_offset));
    return v;
}
// waits until at most n of this wave's LDS reads are still under way (they complete in issue order)
__device__ __forceinline__ void wait_lds_reads(int n) {
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(n));
}

template <int U, int MTW, int EPI>
__global__ __launch_bounds__(256, 1) void k_gemm_big(const u32x4 *__restrict__ Wp, const u32x4 *__restrict__ Xf,
                                                     float *__restrict__ P, int Npad, int K, int S, int MTT, int n_mt,
                                                     int n_pm, GemmEpi e) {
    extern __shared__ __attribute__((aligned(16))) unsigned char bsm[];
    typedef __attribute__((address_space(3))) void lds_void;
    typedef const __attribute__((address_space(1))) void glb_void;
    constexpr int XT = 2 * MTW * 64;       // 16-byte units of one 64-k tile of activations: [s][m][64]
    constexpr int XD = 4;                  // activation fragments read from LDS ahead of their use
    constexpr int NP = 2 * MTW;            // (s, m) fragments per tile
    constexpr int NXF = (NP + 3) / 4;      // one-KiB pieces of an activation tile a wave copies into LDS
    constexpr int NOPS = NXF + 1 + 2 * U;  // load steps of a wave per tile: its share of X(t+1), the touches, then W(t+3)
    u32x4 *xs = (u32x4 *)bsm;              // [2][XT]
    // the wave number as a scalar: everything derived from it (which weight rows, which pieces of the activation
    // tile this wave fetches, where they land in LDS) is then computed once per wave, not per lane
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l = threadIdx.x & 63, li = l & 15, lg = l >> 4;
    const int nunits = Npad / 16, ngrp = (nunits + 4 * U - 1) / (4 * U);
    int bid = blockIdx.x;
    const int g = bid % ngrp; bid /= ngrp;
    const int pm = bid % n_pm, sp = bid / n_pm;
    const int mt0 = pm * MTW, mt_cnt = min(MTW, n_mt - mt0);
    const int nkt = K / 64;
    const int kt0 = split_begin(sp, nkt, S), kt1 = split_begin(sp + 1, nkt, S);
    const int ug0 = (g * 4 + wave) * U;
    // Addresses are a kernel argument plus a 32-bit byte offset (the launcher checks that both operands are
    // smaller than 4 GiB): the per-lane part of the offset is computed once, the per-tile part is one addition.
    const char *Wb = (const char *)Wp, *Xb = (const char *)Xf;
    unsigned woff[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
        const int ug = min(ug0 + j, nunits - 1);
        woff[j] = (unsigned)(((size_t)(ug >> 2) * nkt * 8 + (ug & 3) * 2) * 1024) + l * 16;
    }
    u32x4 wr[4][U][2];   // ring of weight fragments: tile t lives in slot (t - kt0) % 4
    // weight fragment (j, s) of tile kt into ring slot `slot`
    auto wload1 = [&](int q, int kt, int slot) {
        const int j = q >> 1, s = q & 1;
        wr[slot][j][s] = __builtin_nontemporal_load((const u32x4 *)(Wb + (woff[j] + (unsigned)kt * 8192u + s * 1024u)));
    };
    // The 2 * MTW one-KiB pieces (s, m) of an activation tile are dealt to the waves in turn; piece i of this wave
    // for tile kt goes to LDS buffer b (tiles past the last one re-read it: computed, never stored).  Every wave
    // issues the same number of copies, which the waits below count on: where the pieces do not divide by four,
    // the last one is copied by more than one wave (same bytes to the same place).
    const unsigned xstride = (unsigned)MTT * 2048u;   // bytes of the activation fragments of one 64-k tile
    auto xfill1 = [&](int i, int kt, int b) {
        const int f = min(wave + 4 * i, NP - 1), m = f % MTW, s = f / MTW;
        const unsigned off = (unsigned)(s * MTT + min(mt0 + m, MTT - 1)) * 1024u + (unsigned)kt * xstride;
        u32x4 *dst = xs + (size_t)b * XT + (s * MTW + m) * 64;   // wave-uniform; lane i lands at dst + i
        __builtin_amdgcn_global_load_lds((glb_void *)(Xb + (off + (unsigned)l * 16u)), (lds_void *)dst, 16, 0, 0);
    };
    // The activation fragments of a 64-k tile are two runs of MTW KiB (one per k half).  They are touched two
    // tiles ahead with one 4-byte load per 128-byte line (one line per lane and run, lanes past the end repeat the
    // last line), so that the copy into LDS one tile later finds them in L2 instead of waiting for HBM.  The
    // touches are loads to LDS as well, into 256 bytes per wave behind the tile buffers that nobody reads: a load
    // into a register nobody reads would have that register handed to another value while the load is under way.
    const int pf_lines = min(MTW, MTT - mt0) * 8;
    const unsigned pf_off = (unsigned)mt0 * 1024u + (unsigned)min((int)threadIdx.x, pf_lines - 1) * 128u;
    unsigned char *pf_sink = bsm + (size_t)2 * XT * 16 + wave * 256;
    // EPI_SWIGLU: RMSNorm's scale of each of the workgroup's rows (from the per-chunk sums of squares of the input
    // rows), one row per thread, fetched now and parked in LDS behind the sinks until the epilogue
    float *rsc_s = (float *)(bsm + (size_t)2 * XT * 16 + 4 * 256);   // [MTW * 16]
    int *rslot_s = (int *)(rsc_s + MTW * 16), *rbat_s = rslot_s + MTW * 16;   // EPI_QKV: cache slot and sequence of a row
    if (EPI == EPI_QKV && threadIdx.x < MTW * 16) {
        const int row = mt0 * 16 + threadIdx.x;
        const bool ok = row < e.rows;
        rslot_s[threadIdx.x] = ok ? e.meta.row_slot[row] : 0;
        rbat_s[threadIdx.x] = ok ? e.meta.row_b[row] : 0;
    }
    if (EPI != EPI_PARTIAL && threadIdx.x < MTW * 16) {
        const int row = mt0 * 16 + threadIdx.x;
        float tot = 0.f;
        if (e.sums && row < e.rows) {
            for (int c0 = 0; c0 < e.nparts; c0 += 8) {
                float part[8];
#pragma unroll
                for (int c = 0; c < 8; ++c)
                    part[c] = c0 + c < e.nparts ? e.sums[(size_t)(c0 + c) * e.srows + row] : 0.f;
#pragma unroll
                for (int c = 0; c < 8; ++c) tot += part[c];
            }
        }
        rsc_s[threadIdx.x] = e.sums ? 1.0f / sqrtf(tot / (float)e.Kn + e.eps) : 1.f;
    }
    auto xtouch = [&](int kt) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
            __builtin_amdgcn_global_load_lds((glb_void *)(Xb + (pf_off + (unsigned)(2 * kt + s) * ((unsigned)MTT * 1024u))),
                                             (lds_void *)pf_sink, 4, 0, 0);
    };
    f32x4 acc[U][MTW];
#pragma unroll
    for (int j = 0; j < U; ++j)
#pragma unroll
        for (int m = 0; m < MTW; ++m) acc[j][m] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // Memory operations complete in issue order.  Issued before the loop: W(kt0), W(kt0+1), W(kt0+2), X(kt0), all
    // awaited.  The iteration of tile t issues this wave's pieces of X(t+1) and then W(t+3) (into the ring slot
    // tile t-1 has left), one load between the MFMAs of every (s, m) pair, so that neither the address arithmetic
    // nor the issue of the loads holds the matrix pipe up.  At the top of the next iteration only those 2 U weight
    // loads may still be under way: X(t+1) and every older load have landed, and a weight tile has two iterations
    // to arrive from HBM.  Between the two come the two touches of X(t+3), which may stay under way as well (X(t+1),
    // issued before them, has landed all the same).  Past the last tile the same loads are issued again for the last tile, so that the count the wait
    // relies on stays the same.
    constexpr int VM = 2 * U + 2;
    constexpr int WAIT_BUT_NEWEST = (VM & 15) | (7 << 4) | (15 << 8) | ((VM >> 4) << 14);   // s_waitcnt vmcnt(2U + 2)
    const int last = kt1 - 1;
    if (kt0 < kt1) {
#pragma unroll
        for (int q = 0; q < 2 * U; ++q) wload1(q, kt0, 0);
#pragma unroll
        for (int q = 0; q < 2 * U; ++q) wload1(q, min(kt0 + 1, last), 1);
#pragma unroll
        for (int q = 0; q < 2 * U; ++q) wload1(q, min(kt0 + 2, last), 2);
#pragma unroll
        for (int i = 0; i < NXF; ++i) xfill1(i, kt0, 0);
        xtouch(min(kt0 + 1, last));
        xtouch(min(kt0 + 2, last));
        __builtin_amdgcn_s_waitcnt(0);
    }
    // One 64-k tile; p = (tt - kt0) % 4 says where it lives in the weight ring and the LDS buffers.  The tiles come
    // in groups of four with no decisions in between (so that the compiler's view of which loads are under way
    // stays exact from one group to the next), followed by up to three tiles of a last, partial group.
    // The tiles of the last, partial group wait for every load instead: the weight loads they would issue feed
    // no later tile, the compiler drops them, and "all but the newest 2 U + 2" would then let copies of the
    // activation tile pass that have not landed.
    constexpr int WAIT_ALL_LOADS = (7 << 4) | (15 << 8);   // s_waitcnt vmcnt(0)
    auto tile = [&](int tt, auto pc, auto lastgroup) __attribute__((always_inline)) {
        constexpr int p = decltype(pc)::value;
        // nothing is under way before the first tile
        __builtin_amdgcn_s_waitcnt(decltype(lastgroup)::value ? WAIT_ALL_LOADS : WAIT_BUT_NEWEST);
        // every wave's part of X(tt) is in LDS; nobody still reads the other buffer.  A bare barrier instruction
        // (the waits it needs are the ones above), fenced for the compiler so that no LDS access crosses it
        asm volatile("s_barrier" ::: "memory");
        // The activation fragments come from LDS through a ring of XD + 1 registers, read XD fragments ahead
        // of the MFMAs that use them, because an LDS read takes longer than the U MFMAs of one fragment.
        // Reads and waits are written out as instructions: LDS reads complete in issue order,
        // so "at most XD - 1 reads still under way" says exactly that the fragment about to be used has
        // arrived, which the compiler's own bookkeeping rounds down to "none under way" for operands of the
        // MFMA statement above.  The results of such a read must stay where they are until that wait, which
        // holds as long as the kernel does not spill (one workgroup per compute unit: 512 registers a lane).
        // The scheduling fences keep the statements in the order written: other instructions go between
        // the MFMAs, a few at a time, where the matrix pipe is busy anyway.
        lds_u32x4 *xb = (lds_u32x4 *)(xs + (size_t)(p & 1) * XT + l);
        const int ktx = min(tt + 1, last), ktw = min(tt + 3, last);
        u32x4 xr[XD + 1];
#pragma unroll
        for (int i = 0; i < XD; ++i) xr[i] = lds_read16(xb, i * 1024);
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int s = i / MTW, m = i % MTW;
            wait_lds_reads(NP - 1 - i < XD - 1 ? NP - 1 - i : XD - 1);   // reads issued after fragment i's
            const f16x8 xv = __builtin_bit_cast(f16x8, xr[i % (XD + 1)]);
            __builtin_amdgcn_sched_barrier(0);
            mfma_acc(acc[0][m], __builtin_bit_cast(f16x8, wr[p][0][s]), xv);
            __builtin_amdgcn_sched_barrier(0);
            if (i + XD < NP) xr[(i + XD) % (XD + 1)] = lds_read16(xb, (i + XD) * 1024);
            __builtin_amdgcn_sched_barrier(0);
            mfma_acc(acc[1][m], __builtin_bit_cast(f16x8, wr[p][1][s]), xv);
            __builtin_amdgcn_sched_barrier(0);
            // this fragment's share of the tile's global loads: X pieces first, then W fragments
#pragma unroll
            for (int q = i * NOPS / NP; q < (i + 1) * NOPS / NP; ++q) {
                if (q < NXF) xfill1(q, ktx, (p + 1) & 1);
                else if (q == NXF) xtouch(ktw);
                else wload1(q - NXF - 1, ktw, (p + 3) & 3);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 2; j < U; ++j) mfma_acc(acc[j][m], __builtin_bit_cast(f16x8, wr[p][j][s]), xv);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    int t = kt0;
    for (; t + 4 <= kt1; t += 4) {
        tile(t, std::integral_constant<int, 0>{}, std::false_type{});
        tile(t + 1, std::integral_constant<int, 1>{}, std::false_type{});
        tile(t + 2, std::integral_constant<int, 2>{}, std::false_type{});
        tile(t + 3, std::integral_constant<int, 3>{}, std::false_type{});
    }
    if (t < kt1) tile(t, std::integral_constant<int, 0>{}, std::true_type{});
    if (t + 1 < kt1) tile(t + 1, std::integral_constant<int, 1>{}, std::true_type{});
    if (t + 2 < kt1) tile(t + 2, std::integral_constant<int, 2>{}, std::true_type{});
    {
        f32x4 *t = &acc[0][0];
        constexpr int NT = U * MTW;
        static_assert(NT >= 4, "at least four accumulator tiles");
#pragma unroll
        for (int i = 0; i + 4 <= NT; i += 4) {
            if (i == 0) mfma_settle<true>(t[i], t[i + 1], t[i + 2], t[i + 3]);
            else mfma_settle<false>(t[i], t[i + 1], t[i + 2], t[i + 3]);
        }
        if (NT % 4) mfma_settle<false>(t[NT - 4], t[NT - 3], t[NT - 2], t[NT - 1]);   // the last tiles (again)
    }
    __syncthreads();
    if (EPI == EPI_PARTIAL) {
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (ug0 + j >= nunits) continue;
#pragma unroll
            for (int m = 0; m < MTW; ++m) {
                if (m < mt_cnt) {
                    const int row = (mt0 + m) * 16 + li, n = (ug0 + j) * 16 + 4 * lg;
                    *(f32x4 *)(P + ((size_t)sp * (MTT * 16) + row) * Npad + n) = acc[j][m];
                }
            }
        }
    } else if (EPI == EPI_QKV) {
        // One K split.  RMSNorm's row scale, then per lane four columns of one activation row: of V as they are;
        // of Q and K two rotary pairs (the weight rows interleave dimension i and i + head_dim/2), rotated with
        // the row's cos/sin; K and V rows go to the bf16 cache at the row's slot, Q as hi/lo fragments of the
        // attention kernel, times log2(e)/sqrt(head_dim).
        const int half = e.DH / 2;
#pragma unroll
        for (int m = 0; m < MTW; ++m) {
            const int row = (mt0 + m) * 16 + li;
            if (m >= mt_cnt || row >= e.rows) continue;
            const float rsc = rsc_s[m * 16 + li];
            const int slot = rslot_s[m * 16 + li], bat = rbat_s[m * 16 + li];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int n = (ug0 + j) * 16 + 4 * lg;
                if (ug0 + j >= nunits || n >= 3 * e.H) continue;
                const f32x4 v = acc[j][m] * rsc;
                const int which = n / e.H, nn = n % e.H, h = nn / e.DH, r = nn % e.DH;
                const size_t o = (((size_t)bat * e.n_heads + h) * e.cap + slot) * e.DH;
                if (which == 2) {
                    const uint32_t lo = f2bf(v[0]) | (f2bf(v[1]) << 16), hi = f2bf(v[2]) | (f2bf(v[3]) << 16);
                    *(u64_pair *)(e.vc + o + r) = u64_pair{lo, hi};
                    continue;
                }
                const int dd = r >> 1;   // even: the lane holds pairs dd and dd + 1
                const float c0 = e.meta.rope_cos[(size_t)row * half + dd], s0 = e.meta.rope_sin[(size_t)row * half + dd];
                const float c1 = e.meta.rope_cos[(size_t)row * half + dd + 1], s1 = e.meta.rope_sin[(size_t)row * half + dd + 1];
                const float a0 = v[0] * c0 - v[1] * s0, b0 = v[1] * c0 + v[0] * s0;
                const float a1 = v[2] * c1 - v[3] * s1, b1 = v[3] * c1 + v[2] * s1;
                if (which == 1) {
                    *(uint32_t *)(e.kc + o + dd) = f2bf(a0) | (f2bf(a1) << 16);
                    *(uint32_t *)(e.kc + o + half + dd) = f2bf(b0) | (f2bf(b1) << 16);
                } else {
                    const int i = row - bat * e.rows_per_seq;   // row of its sequence
                    uint32_t *qt = e.qf + ((((size_t)bat * e.n_heads + h) * e.MTQ + (i >> 4)) * (e.DH / 32)) * 2 * 64 * 4;
                    const float y[4] = {a0 * e.qscale, a1 * e.qscale, b0 * e.qscale, b1 * e.qscale};
#pragma unroll
                    for (int z = 0; z < 2; ++z) {
                        const int d = dd + z * half;
                        const HiLo pr = split_pair(y[2 * z], y[2 * z + 1]);
                        uint32_t *dst = qt + (((size_t)(d >> 5) * 2) * 64 + (i & 15) + 16 * ((d & 31) >> 3)) * 4 + ((d & 7) >> 1);
                        dst[0] = pr.hi;
                        dst[64 * 4] = pr.lo;
                    }
                }
            }
        }
    } else {
        // EPI_SWIGLU (one K split): the weight rows interleave gate and up, so a lane's four columns are (gate, up)
        // of two features of one activation row.  RMSNorm's row scale (from the per-chunk sums of squares of the
        // input rows) is applied, then SiLU(gate) * up, stored as fragments of the down projection's input.
#pragma unroll
        for (int m = 0; m < MTW; ++m) {
            const int row = (mt0 + m) * 16 + li;
            if (m >= mt_cnt || row >= e.rows) continue;
            const float rsc = rsc_s[m * 16 + li];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int n = (ug0 + j) * 16 + 4 * lg, f0 = n >> 1;
                if (ug0 + j >= nunits || f0 >= e.F) continue;
                const f32x4 v = acc[j][m] * rsc;
                const float g0 = v[0], g1 = v[2];
                const float y0 = g0 / (1.0f + __expf(-g0)) * v[1], y1 = g1 / (1.0f + __expf(-g1)) * v[3];
                const int ks = f0 >> 5, lane = li + 16 * ((f0 & 31) >> 3);
                e.Xo[(((size_t)ks * MTT + (mt0 + m)) * 64 + lane) * 4 + ((f0 & 7) >> 1)] = half_pair(y0, y1);
            }
        }
    }
}

// Sums of split-K partials.  Loads are issued in batches (16 vector loads / 24 scalar loads in
// flight) so that a sum costs one or two memory round trips; the order of the additions is fixed.
__device__ __forceinline__ float psum(const float *P, int S, int Mp, int ld, int row, int col) {
    const float *p = P + (size_t)row * ld + col;
    const size_t stride = (size_t)Mp * ld;
    float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f;
    int s = 0;
    for (; s + 4 <= S; s += 4) {
        v0 += p[(size_t)s * stride];
        v1 += p[(size_t)(s + 1) * stride];
        v2 += p[(size_t)(s + 2) * stride];
        v3 += p[(size_t)(s + 3) * stride];
    }
    for (; s < S; ++s) v0 += p[(size_t)s * stride];
    return (v0 + v1) + (v2 + v3);
}

// N sums at once: element (row, col[i]) for i < N
template <int N>
__device__ __forceinline__ void psum_n(const float *P, int S, int Mp, int ld, int row, const int *col, float *out) {
    const float *p = P + (size_t)row * ld;
    const size_t stride = (size_t)Mp * ld;
    float acc[N];
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = 0.f;
    int s = 0;
    for (; s + 4 <= S; s += 4) {
        float t[4][N];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < N; ++i) t[u][i] = p[(size_t)(s + u) * stride + col[i]];
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] += (t[0][i] + t[1][i]) + (t[2][i] + t[3][i]);
    }
    for (; s < S; ++s)
#pragma unroll
        for (int i = 0; i < N; ++i) acc[i] += p[(size_t)s * stride + col[i]];
#pragma unroll
    for (int i = 0; i < N; ++i) out[i] = acc[i];
}

// 8 consecutive columns (col % 8 == 0) of the summed partials of a row
__device__ __forceinline__ void psum8(const float *P, int S, int Mp, int ld, int row, int col, float *v) {
    const f32x4 *src = (const f32x4 *)(P + (size_t)row * ld + col);
    const size_t stride = (size_t)Mp * ld / 4;   // in f32x4 units
    f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
    int s = 0;
    for (; s + 8 <= S; s += 8) {
        f32x4 a[8], b[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            a[u] = src[(size_t)(s + u) * stride];
            b[u] = src[(size_t)(s + u) * stride + 1];
        }
        lo += ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
        hi += ((b[0] + b[1]) + (b[2] + b[3])) + ((b[4] + b[5]) + (b[6] + b[7]));
    }
    for (; s + 4 <= S; s += 4) {
        const f32x4 a0 = src[(size_t)s * stride], b0 = src[(size_t)s * stride + 1];
        const f32x4 a1 = src[(size_t)(s + 1) * stride], b1 = src[(size_t)(s + 1) * stride + 1];
        const f32x4 a2 = src[(size_t)(s + 2) * stride], b2 = src[(size_t)(s + 2) * stride + 1];
        const f32x4 a3 = src[(size_t)(s + 3) * stride], b3 = src[(size_t)(s + 3) * stride + 1];
        lo += (a0 + a1) + (a2 + a3);
        hi += (b0 + b1) + (b2 + b3);
    }
    for (; s < S; ++s) {
        lo += src[(size_t)s * stride];
        hi += src[(size_t)s * stride + 1];
    }
    v[0] = lo[0]; v[1] = lo[1]; v[2] = lo[2]; v[3] = lo[3];
    v[4] = hi[0]; v[5] = hi[1]; v[6] = hi[2]; v[7] = hi[3];
}

// store 8 consecutive k of row m (k0 % 8 == 0) into the GEMM input fragments
__device__ __forceinline__ void store_frag8(u32x4 *Xf, int MT, int m, int k0, const float *y) {
    const int ks = k0 >> 5, lane = (m & 15) + 16 * ((k0 & 31) >> 3), mt = m >> 4;
    Xf[(size_t)(ks * MT + mt) * 64 + lane] = half8(y);
}

// RMSNorm row scale from the per-chunk sums of squares a fold left: 1/sqrt(mean(x^2) + eps).
// sums == nullptr: no normalisation pending, scale 1.
struct RowScale {
    const float *sums;   // [nparts][srows]
    int nparts, srows, K;
    float eps;
};
__device__ __forceinline__ float row_scale(const RowScale &rs, int row) {
    if (!rs.sums) return 1.f;
    float tot = 0.f;
    for (int c = 0; c < rs.nparts; ++c) tot += rs.sums[(size_t)c * rs.srows + row];
    return 1.0f / sqrtf(tot / (float)rs.K + rs.eps);
}

// A packed weight matrix from bf16 to fp16, in place, eight values (16 bytes) a thread and step.  Every bf16 value
// of magnitude 2^-24 .. 65504 has an exact fp16 image (at most eight significant bits, fp16 holds eleven, fewer
// below 2^-14); smaller ones round to the nearest multiple of 2^-24, larger ones become infinite.
__global__ __launch_bounds__(256) void k_weights_to_f16(u32x4 *w, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) {
        const u32x4 v = w[i];
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
        uint32_t o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            o[q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(
                                                    (f32x2){__uint_as_float(d[q] << 16), __uint_as_float(d[q] & 0xFFFF0000u)}, f16x2));
        w[i] = (u32x4){o[0], o[1], o[2], o[3]};
    }
}

// ---------------------------------------------------------------------------------------------
// Fold: v = (mode 1: x +) sum of partials (mode 0: x as is); x <- v (modes 1, 2); optionally the
// fragments of gain * v (gain == nullptr: of v) for the next GEMM, and the sum of squares of
// each 512-column chunk to sums[chunk][m].  RMSNorm is linear in the row scale, so the GEMM runs
// on gain * v and its consumer multiplies by row_scale().  grid (ceil(N/512), M), 64 threads x 8 cols.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_fold(float *x, const float *P, const bf16_t *gain, u32x4 *Xf, int ldx, int S,
                                             int Mp, int ldp, int mode, int N, int MT, float *sums, int srows) {
    const int c = blockIdx.x, m = blockIdx.y, j = (c * 64 + threadIdx.x) * 8;
    float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (j < N) {
        float *xr = x + (size_t)m * ldx + j;
        if (mode != 0) psum8(P, S, Mp, ldp, m, j, v);
        if (mode != 2) {
            const f32x4 a = *(const f32x4 *)xr, b = *(const f32x4 *)(xr + 4);
            v[0] += a[0]; v[1] += a[1]; v[2] += a[2]; v[3] += a[3];
            v[4] += b[0]; v[5] += b[1]; v[6] += b[2]; v[7] += b[3];
        }
        if (mode != 0) {
            *(f32x4 *)xr = (f32x4){v[0], v[1], v[2], v[3]};
            *(f32x4 *)(xr + 4) = (f32x4){v[4], v[5], v[6], v[7]};
        }
        if (Xf) {
            float y[8];
            if (gain) {
                const u32x4 g = *(const u32x4 *)(gain + j);
                const uint32_t gw[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) y[e] = v[e] * bf2f((e & 1) ? (gw[e >> 1] >> 16) : (gw[e >> 1] & 0xFFFFu));
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) y[e] = v[e];
            }
            store_frag8(Xf, MT, m, j, y);
        }
    }
    if (!sums) return;
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) ss += v[e] * v[e];
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
    if (threadIdx.x == 0) sums[(size_t)c * srows + m] = ss;
}

// ---------------------------------------------------------------------------------------------
// RoPE + KV append from the QKV partials.  grid (rows, n_heads), block head_dim/2.
// ---------------------------------------------------------------------------------------------
__global__ void k_rope_append_p(const float *P, int S, int Mp, int ldp, RowScale rs, RowMeta meta, bf16_t *qf,
                                bf16_t *kc, bf16_t *vc, int H, int n_heads, int DH, int cap, int rows_per_seq, int MTQ,
                                float qscale) {
    const int r = blockIdx.x, h = blockIdx.y, i = threadIdx.x, half = DH / 2;
    const int b = meta.row_b[r], slot = meta.row_slot[r];
    const float c = meta.rope_cos[(size_t)r * half + i], s = meta.rope_sin[(size_t)r * half + i];
    // W_q and W_k rows are stored pair-interleaved: output 2i of a head is dimension i, 2i + 1 is i + half
    const int cols[6] = {h * DH + 2 * i, h * DH + 2 * i + 1, H + h * DH + 2 * i, H + h * DH + 2 * i + 1,
                         2 * H + h * DH + i, 2 * H + h * DH + half + i};
    float t[6];
    psum_n<6>(P, S, Mp, ldp, r, cols, t);
    const float sc = row_scale(rs, r);
    const float q0 = sc * t[0], q1 = sc * t[1], k0 = sc * t[2], k1 = sc * t[3], v0 = sc * t[4], v1 = sc * t[5];
    // query fragments [b][h][MTQ][DH/32][hi, lo][64 lanes][8]: row ri of the sequence, dimensions i and i + half
    const int ri = r - b * rows_per_seq;
    bf16_t *qt = qf + ((((size_t)b * n_heads + h) * MTQ + (ri >> 4)) * (DH / 32)) * 2 * 64 * 8;
    const float y[2] = {(q0 * c - q1 * s) * qscale, (q1 * c + q0 * s) * qscale};
#pragma unroll
    for (int z = 0; z < 2; ++z) {
        const int d = i + z * half;
        const uint32_t hi = f2bf(y[z]), lo = f2bf(y[z] - bf2f(hi));
        bf16_t *dst = qt + (((size_t)(d >> 5) * 2) * 64 + (ri & 15) + 16 * ((d & 31) >> 3)) * 8 + (d & 7);
        dst[0] = (bf16_t)hi;
        dst[64 * 8] = (bf16_t)lo;
    }
    const size_t o = (((size_t)b * n_heads + h) * cap + slot) * DH;
    kc[o + i] = (bf16_t)f2bf(k0 * c - k1 * s);
    kc[o + half + i] = (bf16_t)f2bf(k1 * c + k0 * s);
    vc[o + i] = (bf16_t)f2bf(v0);
    vc[o + half + i] = (bf16_t)f2bf(v1);
}

// SiLU(gate) * up from the gate/up partials (col 2f = gate, 2f+1 = up), scaled by the pending RMSNorm
// row scale, as fragments (K = F).  grid (ceil(F/8/64), M), 64 threads x 8 outputs
__global__ __launch_bounds__(64) void k_silu_frag(const float *P, int S, int Mp, int ldp, RowScale rs, u32x4 *Xf,
                                                  int MT, int F) {
    const int r = blockIdx.y, g = blockIdx.x * 64 + threadIdx.x;
    if (g >= F / 8) return;
    float gu[16];
    psum8(P, S, Mp, ldp, r, g * 16, gu);
    psum8(P, S, Mp, ldp, r, g * 16 + 8, gu + 8);
    const float sc = row_scale(rs, r);
    float y[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float a = sc * gu[2 * e];
        y[e] = a / (1.0f + __expf(-a)) * (sc * gu[2 * e + 1]);
    }
    store_frag8(Xf, MT, r, g * 8, y);
}

// Medusa residual block: x += SiLU(sum of partials)
__global__ void k_resblock_p(float *x, int ldx, const float *P, int S, int Mp, int ldp, int M, int H) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)M * H) return;
    const int r = (int)(i / H), j = (int)(i % H);
    const float v = psum(P, S, Mp, ldp, r, j);
    x[(size_t)r * ldx + j] += v / (1.0f + __expf(-v));
}

// logits[r][v] = sum of partials for v < V
__global__ void k_reduce_out(const float *P, int S, int Mp, int ldp, float *out, int ldo, int M, int N) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)M * N) return;
    const int r = (int)(i / N), j = (int)(i % N);
    out[(size_t)r * ldo + j] = psum(P, S, Mp, ldp, r, j);
}

// ---------------------------------------------------------------------------------------------
// LM-head epilogue: fold the split-K partials into logits and take the k largest per row
// (descending value, equal values by ascending index) in two stages.
// Stage 1, grid (ceil(V/1024), rows): each block reduces 1024 columns, optionally stores the
// logits, and emits its own k best.  Stage 2, grid (rows): merges the blocks' candidates.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) {
    return v > bv || (v == bv && i < bi);
}

// block-wide arg-best over (v, i); every thread gets the winner.  4 waves.
__device__ __forceinline__ void block_best(float &v, int &i, float *sv, int *si) {
    for (int o = 32; o > 0; o >>= 1) {
        const float v2 = __shfl_xor(v, o);
        const int i2 = __shfl_xor(i, o);
        if (better(v2, i2, v, i)) { v = v2; i = i2; }
    }
    __syncthreads();   // previous round's readers are done with sv/si
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = v; si[threadIdx.x >> 6] = i; }
    __syncthreads();
    v = sv[0]; i = si[0];
#pragma unroll
    for (int w = 1; w < 4; ++w)
        if (better(sv[w], si[w], v, i)) { v = sv[w]; i = si[w]; }
}

__global__ __launch_bounds__(256) void k_topk_stage1(const float *P, int S, int Mp, int ldp, RowScale rs,
                                                     float *logits, int ldl, int V, int k, float *cand_val,
                                                     int *cand_idx) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const int r = blockIdx.y, c = blockIdx.x, tid = threadIdx.x, j0 = c * 1024 + tid * 4;
    float val[4] = {0.f, 0.f, 0.f, 0.f};
    if (j0 < V) {   // ldp is a multiple of 64 and j0 of 4: the four columns exist in P even past V
        for (int s = 0; s < S; ++s) {
            const f32x4 v = *(const f32x4 *)(P + ((size_t)s * Mp + r) * ldp + j0);
            val[0] += v[0]; val[1] += v[1]; val[2] += v[2]; val[3] += v[3];
        }
        const float sc = row_scale(rs, r);
        val[0] *= sc; val[1] *= sc; val[2] *= sc; val[3] *= sc;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (j0 + q >= V) val[q] = -INFINITY;
        else if (logits) logits[(size_t)r * ldl + j0 + q] = val[q];
    }
    unsigned taken = 0;
    for (int it = 0; it < k; ++it) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (!((taken >> q) & 1u) && j0 + q < V && better(val[q], j0 + q, bv, bi)) { bv = val[q]; bi = j0 + q; }
        block_best(bv, bi, sv, si);
        if (bi >= j0 && bi < j0 + 4) taken |= 1u << (bi - j0);
        if (tid == 0) {
            cand_val[((size_t)r * gridDim.x + c) * k + it] = bv;
            cand_idx[((size_t)r * gridDim.x + c) * k + it] = bi;
        }
    }
}

__global__ __launch_bounds__(256) void k_topk_stage2(const float *cand_val, const int *cand_idx, int n_cand, int k,
                                                     int32_t *idx, float *val) {
    __shared__ float sv[4];
    __shared__ int si[4];
    const int r = blockIdx.x, tid = threadIdx.x;
    // each thread owns candidates tid, tid+256, ... (at most 4: n_cand <= 1024)
    float cv[4];
    int ci[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int a = tid + 256 * q;
        cv[q] = a < n_cand ? cand_val[(size_t)r * n_cand + a] : -INFINITY;
        ci[q] = a < n_cand ? cand_idx[(size_t)r * n_cand + a] : 0x7fffffff;
    }
    for (int it = 0; it < k; ++it) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (ci[q] != 0x7fffffff && better(cv[q], ci[q], bv, bi)) { bv = cv[q]; bi = ci[q]; }
        block_best(bv, bi, sv, si);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (ci[q] == bi) ci[q] = 0x7fffffff;   // token ids are unique among the candidates
        if (tid == 0) {
            idx[(size_t)r * k + it] = bi;
            if (val) val[(size_t)r * k + it] = bv;
        }
    }
}

inline int cdiv(size_t a, size_t b) { return (int)((a + b - 1) / b); }

template <int U, int MT, int RS, int NW, int PF, int EPI>
void launch_gemm_rows(hipStream_t st, const void *Wp, const void *Xf, int Npad, int K, int S, const GemmEpi &e,
                      hipEvent_t ev_start, hipEvent_t ev_stop) {
    const size_t sm = (size_t)(gemm_rows_tree(U, MT, NW) ? NW / 2 : NW) * U * MT * 64 * 16 + (EPI == EPI_QKV ? (size_t)MT * RS * 16 * U * 8 * 2 * 4 : 0);
    static bool done = false;
    if (!done) {
        (void)hipFuncSetAttribute((const void *)k_gemm_rows<U, MT, RS, NW, PF, EPI>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
        done = true;
    }
    const dim3 grid(((Npad / 16 + U - 1) / U) * S);
    if (ev_start || ev_stop)
        hipExtLaunchKernelGGL((k_gemm_rows<U, MT, RS, NW, PF, EPI>), grid, dim3(64 * NW), sm, st, ev_start, ev_stop, 0,
                              (const u32x4 *)Wp, (const u32x4 *)Xf, Npad, K, S, e);
    else
        k_gemm_rows<U, MT, RS, NW, PF, EPI><<<grid, 64 * NW, sm, st>>>((const u32x4 *)Wp, (const u32x4 *)Xf, Npad, K, S,
                                                                      e);
}

// MTT = 1, 2 or 4 activation tiles
template <int U, int EPI>
void dispatch_gemm_rows_u(hipStream_t st, const void *Wp, const void *Xf, int Npad, int K, int MTT, int S,
                          const GemmEpi &e, hipEvent_t ev_start, hipEvent_t ev_stop) {
    // tiles in flight per wave: two, or one where the registers do not hold a second (four tiles with more than
    // four groups)
    if (MTT == 1) launch_gemm_rows<U, 1, 1, 8, 2, EPI>(st, Wp, Xf, Npad, K, S, e, ev_start, ev_stop);
    else if (MTT == 2) launch_gemm_rows<U, 2, 1, 8, 2, EPI>(st, Wp, Xf, Npad, K, S, e, ev_start, ev_stop);
    else launch_gemm_rows<U, 4, 1, 8, (U <= 4 ? 2 : 1), EPI>(st, Wp, Xf, Npad, K, S, e, ev_start, ev_stop);
}

// 16-row groups per workgroup for an S = 1 launch over Npad rows: the smallest supported count that covers the
// rows with at most one workgroup per compute unit (KOALA_GEMM_U forces a count, for tests and tuning)
int rows_units(int Npad, int n_cu) {
    static const int forced = getenv("KOALA_GEMM_U") ? atoi(getenv("KOALA_GEMM_U")) : 0;
    static const int sup[4] = {3, 4, 6, 7};
    for (int u : sup)
        if (forced == u) return u;
    const int units = Npad / 16;
    for (int u : sup)
        if ((units + u - 1) / u <= n_cu) return u;
    return sup[3];
}

template <int EPI>
void dispatch_gemm_rows(hipStream_t st, const void *Wp, const void *Xf, int Npad, int K, int MTT, int U,
                        const GemmEpi &e, hipEvent_t ev_start, hipEvent_t ev_stop) {
    switch (U) {
    case 3: dispatch_gemm_rows_u<3, EPI>(st, Wp, Xf, Npad, K, MTT, 1, e, ev_start, ev_stop); break;
    case 4: dispatch_gemm_rows_u<4, EPI>(st, Wp, Xf, Npad, K, MTT, 1, e, ev_start, ev_stop); break;
    case 6: dispatch_gemm_rows_u<6, EPI>(st, Wp, Xf, Npad, K, MTT, 1, e, ev_start, ev_stop); break;
    default: dispatch_gemm_rows_u<7, EPI>(st, Wp, Xf, Npad, K, MTT, 1, e, ev_start, ev_stop); break;
    }
}

}  // namespace

// =====================================================================================================
namespace kb {

// tuning knobs from the environment, read once
static int env_int(const char *name, int fallback) {
    const char *e = getenv(name);
    return e && atoi(e) > 0 ? atoi(e) : fallback;
}
static bool wide_passes() {
    static const bool on = !(getenv("KOALA_GEMM_WIDE") && atoi(getenv("KOALA_GEMM_WIDE")) == 0);
    return on;
}

int gemm_splits(int Npad, int K, int MTT) {
    static const int target = env_int("KOALA_GEMM_WGS", 384);
    static const int smax_env = std::min(16, env_int("KOALA_GEMM_SMAX", 16));
    const int nwb = (Npad / 64 + 3) / 4, nch = K / 128;
    const int smax = std::min(smax_env, nch);
    if (MTT >= 8 && wide_passes()) {
        // passes of eight tiles: one 512-thread workgroup per CU is resident, so the grid runs in rounds of 256
        // (a chip of another size would want its CU count here); take the smallest split whose last round is
        // at least 90 % full, else the fullest; at most 8 splits (more splits mean more
        // partial-sum traffic, which at hundreds of rows costs more than a part-empty round: measured)
        int best = 1;
        double best_eff = 0.0;
        for (int S = 1; S <= std::min(smax, 8); ++S) {
            const int wgs = nwb * S, rounds = (wgs + 255) / 256;
            const double eff = (double)wgs / (rounds * 256.0);
            if (eff >= 0.9) return S;
            if (eff > best_eff) { best_eff = eff; best = S; }
        }
        return best;
    }
    int S = (target + nwb / 2) / nwb;
    S = S < 1 ? 1 : S;
    S = S > smax ? smax : S;
    return S;
}

// K splits of gemm_rows_partial: about 256 workgroups of 64 weight rows each
int rows_splits(int Npad, int K) {
    static const int target = env_int("KOALA_ROWS_WGS", 256);
    const int nb = Npad / 64, nkt = K / 64;
    int S = (target + nb / 2) / nb;
    S = S < 1 ? 1 : S > 8 ? 8 : S;
    return S > nkt ? nkt : S;
}

static bool g_attr_done[4] = {false, false, false, false};

static RowScale mk_scale(const NormScale &n) { return RowScale{n.sums, n.nparts, n.srows, n.K, n.eps}; }

void gemm_packed(hipStream_t st, const void *Wp, const void *Xf, float *P, int Npad, int K, int MTT, int S,
                 hipEvent_t ev_start, hipEvent_t ev_stop) {
    const int nwb = (Npad / 64 + 3) / 4;
    const dim3 grid(nwb * S);
#define KOALA_GEMM(MTV, RSV, IDX)                                                                                \
    {                                                                                                            \
        const size_t sm = (size_t)2 * 4 * MTV * RSV * 64 * 16;                                                   \
        if (!g_attr_done[IDX]) {                                                                                 \
            (void)hipFuncSetAttribute((const void *)k_gemm_packed<MTV, RSV>,                                     \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);                      \
            g_attr_done[IDX] = true;                                                                             \
        }                                                                                                        \
        if (ev_start || ev_stop) /* events bound to the dispatch itself: they read the kernel's own begin and end */ \
            hipExtLaunchKernelGGL((k_gemm_packed<MTV, RSV>), grid, dim3(256 * RSV), sm, st,                      \
                                  mt0 == 0 ? ev_start : nullptr, mt0 + g >= MTT ? ev_stop : nullptr, 0,          \
                                  (const u32x4 *)Wp, (const u32x4 *)Xf, P, Npad, K, S, nwb, MTT, mt0);           \
        else                                                                                                     \
            k_gemm_packed<MTV, RSV><<<grid, 256 * RSV, sm, st>>>((const u32x4 *)Wp, (const u32x4 *)Xf, P, Npad, K, \
                                                                 S, nwb, MTT, mt0);                              \
    }
    // MTT is 1, 2 or a multiple of 4: up to eight activation tiles per pass over the weights (eight: two waves
    // per weight row block, four tiles each)
    const bool wide = wide_passes();
    for (int mt0 = 0; mt0 < MTT;) {
        const int left = MTT - mt0;
        const int g = left >= 8 && wide ? 8 : left >= 4 ? 4 : left;
        if (g == 1) KOALA_GEMM(1, 1, 0)
        else if (g == 2) KOALA_GEMM(2, 1, 1)
        else if (g == 4) KOALA_GEMM(4, 1, 2)
        else KOALA_GEMM(4, 2, 3)
        mt0 += g;
    }
#undef KOALA_GEMM
}

void gemm_rows_partial(hipStream_t st, const void *Wp, const void *Xf, float *P, int Npad, int K, int MTT, int S,
                       hipEvent_t ev_start, hipEvent_t ev_stop) {
    GemmEpi e{};
    e.P = P;
    dispatch_gemm_rows_u<4, EPI_PARTIAL>(st, Wp, Xf, Npad, K, MTT, S, e, ev_start, ev_stop);
}

void gemm_rows_qkv(hipStream_t st, const void *Wp, const void *Xf, int K, int MTT, const NormScale &ns, int rows,
                   int rows_per_seq, const RowMeta &meta, void *qf, void *kc, void *vc, int H, int n_heads, int head_dim,
                   int cap, int n_cu, hipEvent_t ev_start, hipEvent_t ev_stop) {
    GemmEpi e{};
    e.sums = ns.sums; e.nparts = ns.nparts; e.srows = ns.srows; e.Kn = ns.K; e.eps = ns.eps;
    e.rows = rows; e.meta = meta; e.qf = (uint32_t *)qf; e.kc = (bf16_t *)kc; e.vc = (bf16_t *)vc;
    e.H = H; e.n_heads = n_heads; e.DH = head_dim; e.cap = cap;
    e.rows_per_seq = rows_per_seq; e.MTQ = (rows_per_seq + 15) / 16;
    e.qscale = 1.4426950408889634f / sqrtf((float)head_dim);   // the attention kernel works in powers of two
    dispatch_gemm_rows<EPI_QKV>(st, Wp, Xf, 3 * H, K, MTT, rows_units(3 * H, n_cu), e, ev_start, ev_stop);
}

void gemm_rows_swiglu(hipStream_t st, const void *Wp, const void *Xf, int K, int MTT, const NormScale &ns, int rows,
                      void *Xo, int F, int n_cu, hipEvent_t ev_start, hipEvent_t ev_stop) {
    GemmEpi e{};
    e.sums = ns.sums; e.nparts = ns.nparts; e.srows = ns.srows; e.Kn = ns.K; e.eps = ns.eps;
    e.rows = rows; e.Xo = (uint32_t *)Xo; e.F = F;
    dispatch_gemm_rows<EPI_SWIGLU>(st, Wp, Xf, pad64(2 * F), K, MTT, rows_units(pad64(2 * F), n_cu), e, ev_start,
                                   ev_stop);
}

// Launch shape of gemm_big for `rows` activation rows: how many blocks the activation tiles are cut into (each
// block streams the weights once, with up to 15 tiles per workgroup), weight row groups per wave (3, 4 or 5) and
// K splits.  Every candidate is priced with a small model of the kernel, in cycles: a workgroup's 64-k tiles cost
// their MFMAs plus a fixed amount (barrier, first LDS reads), a workgroup costs its start-up and its stores, the
// launch takes as many rounds as its workgroups need on the chip's compute units (one workgroup each) but at
// least the time to stream the weights once per tile block, and the partial sums of the splits are written once and read once by the kernel that folds them.
BigShape big_shape(int Npad, int K, int rows, int n_cu, bool one_split) {
    BigShape b{};
    b.n_mt = (rows + 15) / 16;
    const int units = Npad / 16, nkt = K / 64;
    // tuning aids, read once: force the tile blocks / the row groups per wave / the K splits
    static const int fpm = getenv("KOALA_BIG_PM") ? atoi(getenv("KOALA_BIG_PM")) : 0;
    static const int fu = getenv("KOALA_BIG_U") ? atoi(getenv("KOALA_BIG_U")) : 0;
    static const int fs = getenv("KOALA_BIG_S") ? atoi(getenv("KOALA_BIG_S")) : 0;
    double best = 1e300;
    const int pm_lo = (b.n_mt + 14) / 15;
    for (int n_pm = pm_lo; n_pm <= std::min(b.n_mt, pm_lo + 3); ++n_pm) {
        if (fpm >= pm_lo && fpm <= b.n_mt && n_pm != fpm && fpm <= pm_lo + 3) continue;
        const int mtw = (b.n_mt + n_pm - 1) / n_pm;
        const int tmpl = mtw <= 8 ? 8 : mtw <= 10 ? 10 : 15;   // activation tiles the kernel is instantiated for
        for (int U = 5; U >= 3; --U) {
            if (U * tmpl > 60) continue;   // the accumulator tiles of a wave must fit the 256 accumulation registers
            if (fu >= 3 && fu <= 5 && fu * tmpl <= 60 && U != fu) continue;
            for (int S = 1; S <= 4 && S <= nkt; ++S) {
                if (one_split ? S != 1 : (fs >= 1 && fs <= 4 && fs <= nkt && S != fs)) continue;
                const int wgs = ((units + 4 * U - 1) / (4 * U)) * n_pm * S, rounds = (wgs + n_cu - 1) / n_cu;
                const double tiles = (double)((nkt + S - 1) / S);
                const double wg = tiles * (32.0 * tmpl * U / 0.8 + 400.0) + 6000.0 + 30.0 * tmpl * U;
                const double partials = S > 1 ? 2.0 * S * (double)rows * Npad * 4.0 / 4.0e12 * 2.2e9 : 0.0;
                const double hbm = (double)n_pm * Npad * K * 2.0 / 5.0e12 * 2.2e9;   // every tile block streams the weights
                const double cost = std::max(rounds * wg, hbm) + partials;
                if (cost < best) { best = cost; b.n_pm = n_pm; b.mtw = mtw; b.U = U; b.S = S; }
            }
        }
    }
    return b;
}

template <int U, int MTW, int EPI>
static void launch_gemm_big(hipStream_t st, const void *Wp, const void *Xf, float *P, int Npad, int K, int MTT,
                            const BigShape &b, const GemmEpi &e, hipEvent_t ev_start, hipEvent_t ev_stop) {
    // two tile buffers + the sink of the touches + the rows' scales, cache slots and sequences
    const size_t sm = (size_t)2 * 2 * MTW * 64 * 16 + 4 * 256 + 3 * MTW * 16 * 4;
    static bool done = false;
    if (!done) {
        (void)hipFuncSetAttribute((const void *)k_gemm_big<U, MTW, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)sm);
        done = true;
    }
    const dim3 grid(((Npad / 16 + 4 * U - 1) / (4 * U)) * b.n_pm * b.S);
    if (ev_start || ev_stop)
        hipExtLaunchKernelGGL((k_gemm_big<U, MTW, EPI>), grid, dim3(256), sm, st, ev_start, ev_stop, 0,
                              (const u32x4 *)Wp, (const u32x4 *)Xf, P, Npad, K, b.S, MTT, b.n_mt, b.n_pm, e);
    else
        k_gemm_big<U, MTW, EPI><<<grid, 256, sm, st>>>((const u32x4 *)Wp, (const u32x4 *)Xf, P, Npad, K, b.S, MTT,
                                                       b.n_mt, b.n_pm, e);
}

template <int EPI>
static void dispatch_gemm_big(hipStream_t st, const void *Wp, const void *Xf, float *P, int Npad, int K, int MTT,
                              const BigShape &b, const GemmEpi &e, hipEvent_t ev_start, hipEvent_t ev_stop) {
#define KOALA_BIG(UV)                                                                                              \
    {                                                                                                              \
        if (b.mtw <= 8) launch_gemm_big<UV, 8, EPI>(st, Wp, Xf, P, Npad, K, MTT, b, e, ev_start, ev_stop);         \
        else if (b.mtw <= 10) launch_gemm_big<UV, 10, EPI>(st, Wp, Xf, P, Npad, K, MTT, b, e, ev_start, ev_stop);  \
        else launch_gemm_big<UV, 15, EPI>(st, Wp, Xf, P, Npad, K, MTT, b, e, ev_start, ev_stop);                   \
    }
    if (b.U == 3) KOALA_BIG(3) else if (b.U == 4) KOALA_BIG(4)
    else if (b.mtw <= 8) launch_gemm_big<5, 8, EPI>(st, Wp, Xf, P, Npad, K, MTT, b, e, ev_start, ev_stop);
    else launch_gemm_big<5, 10, EPI>(st, Wp, Xf, P, Npad, K, MTT, b, e, ev_start, ev_stop);
#undef KOALA_BIG
}

void gemm_big(hipStream_t st, const void *Wp, const void *Xf, float *P, int Npad, int K, int MTT, const BigShape &b,
              hipEvent_t ev_start, hipEvent_t ev_stop) {
    dispatch_gemm_big<EPI_PARTIAL>(st, Wp, Xf, P, Npad, K, MTT, b, GemmEpi{}, ev_start, ev_stop);
}

// QKV projection of many rows with rotary embedding, KV append and query fragments applied to the accumulators:
// `b` must have one K split
void gemm_big_qkv(hipStream_t st, const void *Wp, const void *Xf, int K, int MTT, const BigShape &b, const NormScale &ns,
                  int rows, int rows_per_seq, const RowMeta &meta, void *qf, void *kc, void *vc, int H, int n_heads,
                  int head_dim, int cap, hipEvent_t ev_start, hipEvent_t ev_stop) {
    GemmEpi e{};
    e.sums = ns.sums; e.nparts = ns.nparts; e.srows = ns.srows; e.Kn = ns.K; e.eps = ns.eps;
    e.rows = rows; e.meta = meta; e.qf = (uint32_t *)qf; e.kc = (bf16_t *)kc; e.vc = (bf16_t *)vc;
    e.H = H; e.n_heads = n_heads; e.DH = head_dim; e.cap = cap;
    e.rows_per_seq = rows_per_seq; e.MTQ = (rows_per_seq + 15) / 16;
    e.qscale = 1.4426950408889634f / sqrtf((float)head_dim);
    dispatch_gemm_big<EPI_QKV>(st, Wp, Xf, nullptr, pad64(3 * H), K, MTT, b, e, ev_start, ev_stop);
}

// gate/up projection of many rows with SwiGLU applied to the accumulators: `b` must have one K split
void gemm_big_swiglu(hipStream_t st, const void *Wp, const void *Xf, int K, int MTT, const BigShape &b,
                     const NormScale &ns, int rows, void *Xo, int F, hipEvent_t ev_start, hipEvent_t ev_stop) {
    GemmEpi e{};
    e.sums = ns.sums; e.nparts = ns.nparts; e.srows = ns.srows; e.Kn = ns.K; e.eps = ns.eps;
    e.rows = rows; e.Xo = (uint32_t *)Xo; e.F = F;
    dispatch_gemm_big<EPI_SWIGLU>(st, Wp, Xf, nullptr, pad64(2 * F), K, MTT, b, e, ev_start, ev_stop);
}

void weights_to_f16(hipStream_t st, void *w, size_t n_elements) {
    const size_t n16 = n_elements / 8;
    if (n16 == 0) return;
    const int grid = (int)std::min<size_t>((n16 + 255) / 256, 4096);
    k_weights_to_f16<<<grid, 256, 0, st>>>((u32x4 *)w, n16);
}

void fold(hipStream_t st, float *x, int ldx, const float *P, int S, int Mp, int ldp, int mode, int M, int N,
          const void *gain, void *Xf, int MT, float *sums, int srows) {
    k_fold<<<dim3((N + 511) / 512, M), 64, 0, st>>>(x, P, (const bf16_t *)gain, (u32x4 *)Xf, ldx, S, Mp, ldp, mode, N,
                                                    MT, sums, srows);
}

void rope_append(hipStream_t st, const float *P, int S, int Mp, int ldp, const NormScale &ns, const RowMeta &meta,
                 void *qf, void *kc, void *vc, int rows, int H, int n_heads, int head_dim, int cap, int rows_per_seq) {
    k_rope_append_p<<<dim3(rows, n_heads), head_dim / 2, 0, st>>>(P, S, Mp, ldp, mk_scale(ns), meta, (bf16_t *)qf,
                                                                  (bf16_t *)kc, (bf16_t *)vc, H, n_heads, head_dim, cap,
                                                                  rows_per_seq, (rows_per_seq + 15) / 16,
                                                                  1.4426950408889634f / sqrtf((float)head_dim));
}

void silu_frag(hipStream_t st, const float *P, int S, int Mp, int ldp, const NormScale &ns, void *Xf, int MT, int M,
               int F) {
    k_silu_frag<<<dim3((F / 8 + 63) / 64, M), 64, 0, st>>>(P, S, Mp, ldp, mk_scale(ns), (u32x4 *)Xf, MT, F);
}

void resblock_p(hipStream_t st, float *x, int ldx, const float *P, int S, int Mp, int ldp, int M, int H) {
    k_resblock_p<<<cdiv((size_t)M * H, 256), 256, 0, st>>>(x, ldx, P, S, Mp, ldp, M, H);
}

// cand buffers: rows * ceil(V/1024) * k entries each
void logits_topk(hipStream_t st, const float *P, int S, int Mp, int ldp, const NormScale &ns, float *logits, int ldl,
                 int rows, int V, int k, float *cand_val, int *cand_idx, int32_t *idx, float *val) {
    const int nchunk = (V + 1023) / 1024;
    k_topk_stage1<<<dim3(nchunk, rows), 256, 0, st>>>(P, S, Mp, ldp, mk_scale(ns), logits, ldl, V, k, cand_val,
                                                      cand_idx);
    k_topk_stage2<<<rows, 256, 0, st>>>(cand_val, cand_idx, nchunk * k, k, idx, val);
}

void reduce_out(hipStream_t st, const float *P, int S, int Mp, int ldp, float *out, int ldo, int M, int N) {
    k_reduce_out<<<cdiv((size_t)M * N, 256), 256, 0, st>>>(P, S, Mp, ldp, out, ldo, M, N);
}

}  // namespace kb

// =====================================================================================================
// Tree-masked attention on MFMA (bf16 KV cache; queries arrive as bf16 hi + lo MFMA fragments, already
// multiplied by log2(e)/sqrt(head_dim), written by the QKV projection's epilogue; the softmax is computed
// with powers of two, which is the same function).
//
// grid (nsplit * row groups, n_heads, batch), NWV waves.  The 32-key steps of the sequence's visible key range
// [0, kv_end) are dealt out round-robin over the nsplit workgroups and their waves, each wave keeping an
// online-softmax state (running max, sum, output) for its MT row tiles, merged through LDS at the end.
// Per step and wave:
//   S^T[key][row] = K[key][:] . Q[row][:]   A = K rows straight from the cache (16 B per lane),
//                                            B = Q fragments (hi, lo) from LDS;
//   mask by the row's visible prefix / ancestor bits, online softmax (row max across the 4 lane groups);
//   O^T[d][row] += V^T[d][key] P^T[key][row] B = the probabilities exactly where the S^T tile left them
//                                            (hi + lo), A = V transposed through a per-wave LDS tile.
// The contraction order of the second product is chosen so that no probability moves between lanes:
// slot (lane group g, element e) stands for key 16*(e/4) + 4*g + e%4 of the step.
//
// The key splits of one (sequence, head, row group) are merged inside the kernel: every workgroup writes
// its partial result (output, running max, sum) through to memory, then adds one to a counter; the
// workgroup that finds the counter at nsplit - 1 reads all partial results back, merges them in split
// order (deterministic) and writes the rows as fragments of the O projection's input.  Nobody waits
// for anybody.  The counter is reset by that last workgroup, so it is zero again at the next launch.
// =====================================================================================================
namespace {

// LDS tiles are written and read through different element types; these typedefs keep the
// compiler from assuming the accesses cannot overlap.
typedef unsigned short __attribute__((may_alias)) u16_alias;
struct __attribute__((may_alias)) u64_alias { unsigned int x, y; };

// Partial results cross workgroups (and so, possibly, L2 caches that are not coherent with each other) inside
// one kernel: they are stored and loaded with the sc1 cache policy (agent scope: written through to, and read
// from, memory that every compute unit sees), through buffer instructions bounded by the allocation size.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr int AUX_SC1 = 16;
__device__ __forceinline__ rsrc_t make_rsrc(const void *p, size_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, bytes > 0xFFFFFFF0ull ? (int)0xFFFFFFF0u : (int)bytes,
                                             0x00020000);
}
__device__ __forceinline__ void st_sc1(rsrc_t r, size_t off, f32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), r, (int)off, 0, AUX_SC1);
}
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
__device__ __forceinline__ void st_sc1(rsrc_t r, size_t off, u32x2 v) {
    __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)off, 0, AUX_SC1);
}
__device__ __forceinline__ u32x4 ld4u_sc1(rsrc_t r, size_t off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, AUX_SC1);
}
__device__ __forceinline__ f32x2 half_pair_to_float(uint32_t p) {
    return __builtin_convertvector(__builtin_bit_cast(f16x2, p), f32x2);
}
__device__ __forceinline__ void st_sc1(rsrc_t r, size_t off, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, (int)off, 0, AUX_SC1);
}
__device__ __forceinline__ f32x4 ld4_sc1(rsrc_t r, size_t off) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, AUX_SC1));
}
__device__ __forceinline__ float ld1_sc1(rsrc_t r, size_t off) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, AUX_SC1));
}

// Maximum / sum over the four 16-lane groups of a wave (lanes l, l^16, l^32, l^48), result in every lane.  The
// swap instructions exchange 16-lane (32-lane) blocks between two registers: with the same value in both, one
// result holds every lane's own block pair partner, so each level is one swap and one operation, all in the
// vector unit (a shuffle through LDS costs a round trip there).
__device__ __forceinline__ float lane_groups_max(float x) {
    const auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float lane_groups_sum(float x) {
    const auto q = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(q[0]) + __uint_as_float(q[1]);
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

struct AttnArgs {
    const u32x4 *qf;      // [batch][n_heads][MTQ][KS][hi, lo][64] query fragments
    RowMeta meta;
    const bf16_t *kc, *vc;
    float *o_part, *ml;   // [row][head][split][DH] fp16 averages (in a buffer sized for fp32), [row][head][split][max, sum]
    unsigned opart_bytes, ml_bytes;
    int *counters;        // [batch][n_heads][row groups], zero between launches
    u32x4 *Xf;            // merged output: GEMM input fragments, K = n_heads * DH, MT_out activation tiles
    int MT_out;
    int rows_per_seq, MTQ, n_heads, cap, nsplit, batch, ngroups;
};

// The arguments that the first loads depend on come first and one by one: leading scalar arguments are handed to a
// wave in registers when it starts, the rest (`a`) it fetches itself.
template <int DH, int MT, int NWV>
__global__ __launch_bounds__(64 * NWV) void k_attn_tree(const u32x4 *qf_in, const bf16_t *kc, const bf16_t *vc,
                                                        const int *kv_end_of, int nsplit, int n_heads, int cap,
                                                        int batch, int ngroups, int rows_per_seq, AttnArgs a) {
    constexpr int KS = DH / 32;            // contraction steps over the head dimension
    constexpr int DT = DH / 16;            // 16-wide output tiles over the head dimension
    constexpr int VS = DH * 2 + 32;        // bytes per key row of the V tile in LDS: rows 8 banks apart, so that a
                                           // transposing load's 16 lanes (4 rows x 32 B) hit 32 different banks
    constexpr int LPR = DH / 8;            // lanes that cover one cache row with 16 B each
    constexpr int VI = DH / 16;            // load instructions per 32-key V tile
    constexpr int NTH = 64 * NWV;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ int s_last;
    u32x4 *qf = (u32x4 *)smem;                                   // [MT][KS][2][64]
    unsigned char *vt_all = smem + (size_t)MT * KS * 2 * 64 * 16;  // [NWV waves][32][VS]
    // One workgroup per (key split, head, sequence) and group of MT row tiles (sequences of more than MT*16 rows
    // take several groups, each with its own row tiles over the same keys).  Workgroups go to the chip's eight
    // dies in turn by their index, each die with an L2 of its own: the groups of one (split, head, sequence) get
    // indices 8 apart, so they run on the same die at about the same time and the keys and values they share are
    // fetched from memory once.  Indices past the last item (the grid is padded to whole rounds) do nothing.
    const int items = nsplit * n_heads * batch, MTQ = (rows_per_seq + 15) / 16;
    const int die = blockIdx.x & 7, round = blockIdx.x >> 3;
    const int item = (round / ngroups) * 8 + die, grp = round % ngroups;
    if (item >= items) return;
    const int s = item % nsplit, h = (item / nsplit) % n_heads, mt0 = grp * MT;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // a scalar: so is all that follows from it
    const int l = tid & 63, li = l & 15, lg = l >> 4;
    unsigned char *vt = vt_all + (size_t)wave * 32 * VS;
    // Sequences are taken longest first: a workgroup's run time grows with its sequence's length, and the ones
    // that run longest must not be the ones that start last.  Every wave ranks the batch's lengths itself (lane j
    // holds sequence j's; equal lengths rank by index), and the item's sequence slot picks the one of that rank.
    int b = item / (nsplit * n_heads), kv_end;
    if (batch > 1 && batch <= 64) {
        const int len = l < batch ? kv_end_of[l] : -1;
        int rank = 0;
        for (int j = 0; j < batch; ++j) {
            const int lj = __builtin_amdgcn_readlane(len, j);
            rank += (lj > len || (lj == len && j < l)) ? 1 : 0;
        }
        const uint64_t hit = __builtin_amdgcn_ballot_w64(l < batch && rank == b);
        if (hit) b = (int)__builtin_ctzll(hit);
        kv_end = __builtin_amdgcn_readlane(len, b);
    } else {
        kv_end = kv_end_of[b];
    }

    // everything that does not depend on the key range is requested first: the query fragments and the rows'
    // visibility data
    u32x4 qreg[(MT * KS * 2 * 64 + NTH - 1) / NTH];
#pragma unroll
    for (int i = 0; i < (MT * KS * 2 * 64 + NTH - 1) / NTH; ++i) {
        const int u = tid + i * NTH, mt = u / (KS * 2 * 64);
        qreg[i] = (u < MT * KS * 2 * 64 && mt0 + mt < MTQ)
                      ? qf_in[(((size_t)b * n_heads + h) * MTQ + mt0) * (KS * 2 * 64) + u]
                      : (u32x4){0u, 0u, 0u, 0u};
    }
    int nvis[MT], base[MT];
    uint64_t mask[MT];
    int nvis_min = 0x7fffffff;   // keys below this are visible to every row of the workgroup: no masking there
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int row = (mt0 + mt) * 16 + li;
        const bool ok = row < rows_per_seq;
        const int r = b * rows_per_seq + (ok ? row : 0);
        nvis[mt] = ok ? a.meta.row_nvis[r] : 0;
        base[mt] = ok ? a.meta.row_base[r] : 0;
        mask[mt] = ok ? a.meta.row_mask[r] : 0ull;
        if (ok) nvis_min = min(nvis_min, nvis[mt]);
    }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) nvis_min = min(nvis_min, __shfl_xor(nvis_min, o));
    nvis_min = __builtin_amdgcn_readfirstlane(nvis_min);
    // The 32-key steps of the sequence are dealt out round-robin, first over the key splits and then over the
    // waves: workgroup s, wave w takes steps s + splits * (w + NWV * k) (a step past the end is loaded from clamped
    // rows and unused).
    const int j1 = kv_end;
    const int nsteps = (kv_end + 31) / 32;
    const int tstride = nsplit * NWV;
    const bf16_t *kb = kc + ((size_t)b * n_heads + h) * cap * DH;
    const bf16_t *vb = vc + ((size_t)b * n_heads + h) * cap * DH;
    u32x4 kf[2][KS], vr[VI];
    auto load_step = [&](int st) {
        const int k0 = st * 32;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int key = min(k0 + 16 * j + li, cap - 1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[j][ks] = *(const u32x4 *)(kb + (size_t)key * DH + ks * 32 + 8 * lg);
        }
#pragma unroll
        for (int i = 0; i < VI; ++i) {
            const int key = min(k0 + i * (64 / LPR) + l / LPR, cap - 1);
            vr[i] = *(const u32x4 *)(vb + (size_t)key * DH + (l % LPR) * 8);
        }
    };
    load_step(s + nsplit * wave);
#pragma unroll
    for (int i = 0; i < (MT * KS * 2 * 64 + NTH - 1) / NTH; ++i)
        if (tid + i * NTH < MT * KS * 2 * 64) qf[tid + i * NTH] = qreg[i];

    f32x4 acc_o[MT][DT];
    float m_run[MT], l_run[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        m_run[mt] = -INFINITY;
        l_run[mt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) acc_o[mt][dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();

    for (int st = s + nsplit * wave; st < nsteps; st += tstride) {
        const int k0 = st * 32;
        // ---- S^T = K Q^T
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
                    const bf16x8 ka = __builtin_bit_cast(bf16x8, kf[j][ks]);
                    sc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qh, sc[j][mt], 0, 0, 0);
                    sc[j][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, ql, sc[j][mt], 0, 0, 0);
                }
            }
        // ---- V tile -> LDS (row-major, padded), written as 8-byte halves
        // a step whose 32 keys every row of the workgroup sees (all but the last few of a sequence) needs no masks,
        // no zeroing of rows past the end and no care for rows that have seen nothing yet
        const bool full = k0 + 32 <= nvis_min && k0 + 32 <= j1;
        if (full) {
#pragma unroll
            for (int i = 0; i < VI; ++i) {
                const int kl = i * (64 / LPR) + l / LPR;
                u64_alias *dst = (u64_alias *)(vt + (size_t)kl * VS + (l % LPR) * 16);
                dst[0] = u64_alias{vr[i].x, vr[i].y};
                dst[1] = u64_alias{vr[i].z, vr[i].w};
            }
        } else {
#pragma unroll
            for (int i = 0; i < VI; ++i) {
                const int kl = i * (64 / LPR) + l / LPR;
                u64_alias *dst = (u64_alias *)(vt + (size_t)kl * VS + (l % LPR) * 16);
                const bool in = k0 + kl < j1;   // rows past the end contribute exact zeros (0 * garbage could be NaN)
                dst[0] = in ? u64_alias{vr[i].x, vr[i].y} : u64_alias{0u, 0u};
                dst[1] = in ? u64_alias{vr[i].z, vr[i].w} : u64_alias{0u, 0u};
            }
        }
        if (st + tstride < nsteps) load_step(st + tstride);   // kf / vr are free again: next step's loads overlap the rest
        // ---- mask, online softmax; probabilities stay in place as the B operand (hi, lo)
        bf16x8 ph[MT], pl[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float p[8], v[8];
            float tmax = -INFINITY, psum = 0.f, alpha;
            if (full) {   // same for the whole workgroup
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = sc[e >> 2][mt][e & 3];
                    tmax = fmaxf(tmax, p[e]);
                }
                tmax = lane_groups_max(tmax);
                // scores are in units of log 2 (the queries carry the factor log2(e)): weights are 2^(score - max);
                // the new maximum is finite here, so a row that had seen nothing gets alpha = 2^(-inf) = 0
                const float m_new = fmaxf(m_run[mt], tmax);
                alpha = __builtin_amdgcn_exp2f(m_run[mt] - m_new);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    v[e] = __builtin_amdgcn_exp2f(p[e] - m_new);
                    psum += v[e];
                }
                m_run[mt] = m_new;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int key = k0 + 16 * (e >> 2) + 4 * lg + (e & 3);
                    const unsigned rel = (unsigned)(key - base[mt]);   // negative differences wrap to >= 64
                    const uint32_t half = rel < 32u ? (uint32_t)mask[mt] : (uint32_t)(mask[mt] >> 32);
                    const bool bit = rel < 64u && ((half >> (rel & 31u)) & 1u);
                    const bool vis = key < j1 && (key < nvis[mt] || bit);
                    p[e] = vis ? sc[e >> 2][mt][e & 3] : -INFINITY;
                    tmax = fmaxf(tmax, p[e]);
                }
                tmax = lane_groups_max(tmax);
                const float m_new = fmaxf(m_run[mt], tmax);
                alpha = (m_run[mt] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run[mt] - m_new);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    v[e] = (p[e] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(p[e] - m_new);
                    psum += v[e];
                }
                m_run[mt] = m_new;
            }
            l_run[mt] = l_run[mt] * alpha + psum;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {   // once the maxima have settled nothing is rescaled
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    acc_o[mt][dt][0] *= alpha; acc_o[mt][dt][1] *= alpha;
                    acc_o[mt][dt][2] *= alpha; acc_o[mt][dt][3] *= alpha;
                }
            }
            u32x4 x, c;
            split8(v, x, c);
            ph[mt] = __builtin_bit_cast(bf16x8, x);
            pl[mt] = __builtin_bit_cast(bf16x8, c);
        }
        // ---- O^T += V^T P^T ; A operand: lane (d%16, g), slot e -> key 16*(e/4)+4g+e%4, read from the row-major LDS
        //      tile with the transposing LDS load: in every group of 16 lanes, lane i hands in the address of four
        //      consecutive 16-bit values and receives element i%4 of the lanes 4e + i/4, e = 0..3.  Lane i therefore
        //      points at key row 4g + i/4, columns 16 dt + 4 (i%4) .., and gets keys 4g .. 4g+3 of column 16 dt + i.
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
            const unsigned char *src = vt + (size_t)(4 * lg + (li >> 2)) * VS + dt * 32 + (li & 3) * 8;
            const bf16x4 k0 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)src);
            const bf16x4 k1 = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(src + 16 * VS));
            const bf16x8 va = __builtin_shufflevector(k0, k1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc_o[mt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, ph[mt], acc_o[mt][dt], 0, 0, 0);
                acc_o[mt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pl[mt], acc_o[mt][dt], 0, 0, 0);
            }
        }
    }
    // ---- row sums across the four lane groups
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        l_run[mt] = lane_groups_sum(l_run[mt]);
    }
    // ---- merge the waves through LDS (the Q / V regions are free now) in one round: every wave that had a step
    //      leaves its state there, then each wave combines, for its share of the (row tile, 16 dimensions) pieces,
    //      the states of all of them (in wave order: deterministic) and writes the piece of this split's partial
    //      result through to memory: the softmax average of the split's keys (the output divided by its sum, so
    //      that it is bounded by the values it averages) in fp16, half the bytes that the merging workgroup has to
    //      take in (the merged rows are rounded to fp16 for the O projection anyway), with the running maximum and
    //      the sum beside it.
    float *mo = (float *)smem;                                  // [NWV waves][MT][DT][64][4]
    float *mm = mo + (size_t)NWV * MT * DT * 256;               // [NWV waves][MT][16 rows][max, sum]
    // waves 0 .. nact-1 had at least one step (wave w starts at step s + nsplit * w)
    const int nact = min(NWV, max(0, (nsteps - s + nsplit - 1) / nsplit));
    __syncthreads();
    if (wave < nact) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
                *(f32x4 *)(mo + ((((size_t)wave * MT + mt) * DT + dt) * 64 + l) * 4) = acc_o[mt][dt];
            if (lg == 0) {
                mm[((wave * MT + mt) * 16 + li) * 2 + 0] = m_run[mt];
                mm[((wave * MT + mt) * 16 + li) * 2 + 1] = l_run[mt];
            }
        }
    }
    __syncthreads();
    const rsrc_t ro = make_rsrc(a.o_part, a.opart_bytes), rm = make_rsrc(a.ml, a.ml_bytes);
    for (int p = wave; p < MT * DT; p += NWV) {
        const int mt = p / DT, dt = p % DT;
        float M = -INFINITY;
        for (int w = 0; w < nact; ++w) M = fmaxf(M, mm[((w * MT + mt) * 16 + li) * 2]);
        float L = 0.f;
        f32x4 O = {0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < nact; ++w) {
            const float mw = mm[((w * MT + mt) * 16 + li) * 2], lw = mm[((w * MT + mt) * 16 + li) * 2 + 1];
            const float aw = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - M);
            L += aw * lw;
            O += aw * *(const f32x4 *)(mo + ((((size_t)w * MT + mt) * DT + dt) * 64 + l) * 4);
        }
        const int row = (mt0 + mt) * 16 + li;
        if (row < rows_per_seq) {
            const size_t r = (size_t)b * rows_per_seq + row;
            const size_t o = (((r * n_heads + h) * nsplit + s) * DH) * 2;
            const f32x4 v = O * (L > 0.f ? 1.0f / L : 0.f);
            st_sc1(ro, o + (dt * 16 + 4 * lg) * 2, (u32x2){half_pair(v[0], v[1]), half_pair(v[2], v[3])});
            if (dt == 0 && lg == 0) {
                const size_t pm = (((r * n_heads + h) * nsplit + s) * 2) * 4;
                st_sc1(rm, pm, M);
                st_sc1(rm, pm + 4, L);
            }
        }
    }
    // the partial results were written through (sc1), so nothing of a wave's is left in a cache to be written back:
    // it is enough that every wave's stores have been acknowledged before the counter moves
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (wave == 0) {
        if (l == 0) {
            int *cnt = a.counters + ((size_t)b * n_heads + h) * ngroups + grp;
            const int old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = old == nsplit - 1;
            if (old == nsplit - 1) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();
    if (!s_last) return;
    // ---- the last workgroup of this (sequence, head, row group) merges the splits: one thread per (row, 8 dims)
    for (int u = tid; u < MT * 16 * (DH / 8); u += NTH) {
        const int row = mt0 * 16 + u / (DH / 8), d0 = (u % (DH / 8)) * 8;
        if (row >= rows_per_seq) continue;
        const size_t r = (size_t)b * rows_per_seq + row;
        const size_t ob = ((r * n_heads + h) * nsplit) * DH * 2 + d0 * 2, mb = ((r * n_heads + h) * nsplit) * 2 * 4;
        u32x4 oh[KOALA_NSPLIT_MAX];   // eight fp16 values of the split's average
        float ms[KOALA_NSPLIT_MAX], ls[KOALA_NSPLIT_MAX];
#pragma unroll
        for (int q = 0; q < KOALA_NSPLIT_MAX; ++q) {
            if (q < nsplit) {
                oh[q] = ld4u_sc1(ro, ob + (size_t)q * DH * 2);
                ms[q] = ld1_sc1(rm, mb + q * 8);
                ls[q] = ld1_sc1(rm, mb + q * 8 + 4);
            } else {
                oh[q] = (u32x4){0u, 0u, 0u, 0u};
                ms[q] = -INFINITY;
                ls[q] = 0.f;
            }
        }
        float Mx = -INFINITY;
#pragma unroll
        for (int q = 0; q < KOALA_NSPLIT_MAX; ++q) Mx = fmaxf(Mx, ms[q]);
        float ys[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        float den = 0.f;
#pragma unroll
        for (int q = 0; q < KOALA_NSPLIT_MAX; ++q) {
            // weight of the split's average: its share of the softmax sum
            const float w = (ms[q] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ms[q] - Mx) * ls[q];
            den += w;
            const uint32_t d[4] = {oh[q].x, oh[q].y, oh[q].z, oh[q].w};
#pragma unroll
            for (int z = 0; z < 4; ++z) {
                const f32x2 p = half_pair_to_float(d[z]);
                ys[2 * z] += w * p[0];
                ys[2 * z + 1] += w * p[1];
            }
        }
        const float inv = 1.0f / den;
        float y[8];
#pragma unroll
        for (int z = 0; z < 8; ++z) y[z] = ys[z] * inv;
        store_frag8(a.Xf, a.MT_out, (int)r, h * DH + d0, y);
    }
}

template <int DH, int MT, int NWV>
void launch_attn(hipStream_t st, const AttnArgs &a, int batch) {
    constexpr int KS = DH / 32, DT = DH / 16, VS = DH * 2 + 32;
    const size_t main_b = (size_t)MT * KS * 2 * 64 * 16 + (size_t)NWV * 32 * VS;
    const size_t merge_b = (size_t)NWV * MT * DT * 256 * 4 + (size_t)NWV * MT * 16 * 2 * 4;
    const size_t sm = main_b > merge_b ? main_b : merge_b;
    static bool done = false;
    if (!done) {
        (void)hipFuncSetAttribute((const void *)k_attn_tree<DH, MT, NWV>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)sm);
        done = true;
    }
    AttnArgs b = a;
    b.batch = batch;
    b.ngroups = (a.rows_per_seq + MT * 16 - 1) / (MT * 16);   // row-tile groups per (split, head, sequence)
    const int items = a.nsplit * a.n_heads * batch;
    k_attn_tree<DH, MT, NWV><<<dim3((items + 7) / 8 * 8 * b.ngroups), 64 * NWV, sm, st>>>(
        b.qf, b.kc, b.vc, b.meta.kv_end, b.nsplit, b.n_heads, b.cap, b.batch, b.ngroups, b.rows_per_seq, b);
}

}  // namespace

namespace kb {

// rows_per_seq <= 64.  counters: batch * n_heads * 4 ints, zero before the first launch (the kernel leaves them
// zero).  The merged rows are written as fragments Xf (MT_out activation tiles) of the O projection's input.
void attention_tree(hipStream_t st, const void *qf, const RowMeta &meta, const void *kc, const void *vc, float *o_part,
                    size_t opart_bytes, float *ml, size_t ml_bytes, int *counters, void *Xf, int MT_out, int batch,
                    int rows_per_seq, int n_heads, int head_dim, int cap, int nsplit) {
    AttnArgs a{};
    a.qf = (const u32x4 *)qf; a.meta = meta; a.kc = (const bf16_t *)kc; a.vc = (const bf16_t *)vc;
    a.o_part = o_part; a.ml = ml;
    a.opart_bytes = (unsigned)std::min<size_t>(opart_bytes, 0xFFFFFFF0u);
    a.ml_bytes = (unsigned)std::min<size_t>(ml_bytes, 0xFFFFFFF0u);
    a.counters = counters; a.Xf = (u32x4 *)Xf; a.MT_out = MT_out;
    a.rows_per_seq = rows_per_seq; a.MTQ = (rows_per_seq + 15) / 16; a.n_heads = n_heads; a.cap = cap; a.nsplit = nsplit;
    // up to 16 rows: one row tile per workgroup; more: two (sequences of more than 32 rows take two workgroups
    // per split and head)
    const int MT = rows_per_seq <= 16 ? 1 : 2;
    static const int forced = getenv("KOALA_ATTN_WAVES") ? atoi(getenv("KOALA_ATTN_WAVES")) : 0;   // tuning: 4 or 8
    const int nwv = forced == 4 || forced == 8 ? forced : 8;
#define KOALA_ATT(DHV, MTV) \
    { if (nwv == 8) launch_attn<DHV, MTV, 8>(st, a, batch); else launch_attn<DHV, MTV, 4>(st, a, batch); }
    if (head_dim == 128) {
        if (MT == 1) KOALA_ATT(128, 1) else KOALA_ATT(128, 2)
    } else {
        if (MT == 1) KOALA_ATT(64, 1) else KOALA_ATT(64, 2)
    }
#undef KOALA_ATT
}

}  // namespace kb
