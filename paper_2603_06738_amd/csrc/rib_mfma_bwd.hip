// RIB window attention, backward, on the gfx950 matrix cores (bf16 MFMA, fp32
// accumulation).  Gradient formulas: include/rib_attn.h (chain rule through paper
// Sec. 2.2 and Sec. 3.1 Eq. 5-6).
//
// Two kernels, both free of atomics so that every output is run-to-run identical:
//
//   dkv kernel  -- a workgroup owns 256 keys of one (window, head) unit (64 per
//     wave, held in registers as MFMA B operands) and streams the unit's queries
//     through LDS in tiles of 64.  Per 32x32 block it forms S = Q_aug K_aug^T and
//     dP = dO V^T in the layout where a lane owns a KEY column, so P and dS, packed
//     to bf16, are directly the B operands of dV^T += dO^T P and
//     dK_aug^T += Q_aug^T dS (contractions over queries).
//   dq kernel   -- a workgroup owns 256 queries and streams keys; it forms the
//     TRANSPOSED blocks S^T, dP^T (a lane owns a QUERY column), so dS^T is the B
//     operand of dQ_aug^T += K_aug^T dS^T (contraction over keys).
//
//   In both kernels it is Q_aug that carries scale * log2(e), rounded to bf16 exactly as the
//   forward rounds it, so the recomputed logits are the forward's bit for bit.
//   P is recomputed as exp2(S - LSE) and dS = P (dP - delta).  Neither
//   subtraction costs a vector instruction: -LSE*log2(e), split into a bf16 high
//   and low part, rides in the last two padding columns of Q_aug against ones in
//   K_aug, and -delta rides the same way in the padding of dO against ones in V,
//   so the matrix cores deliver S - LSE and dP - delta directly.
//
//   The last r columns of dQ_aug / dK_aug are this unit's contribution to dF_q /
//   dF_k (Sec. 3.1: the RIB features are shared by all windows); they go to a
//   per-unit fp32 scratch and are summed over windows in a fixed order afterwards.

#include "rib_common.h"

namespace rib {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kT = 64;                 // tokens per staged tile
constexpr int kTS = kT + 8;            // bf16 per row of a transposed tile
constexpr int kWaves = 4;
constexpr int kNT = kWaves * 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    bf16x2 v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float lo_bf16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_bf16(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
// x as a bf16 pair (hi, lo) with hi + lo == x to ~2^-17 relative
__device__ __forceinline__ uint32_t split_bf16(float x)
{
    bf16x2 v;
    v[0] = (__bf16)x;
    v[1] = (__bf16)(x - (float)v[0]);
    return __builtin_bit_cast(uint32_t, v);
}

// Column of token kappa (0..63) in a transposed tile: inside each group of 16 the
// order in which the 32x32 accumulator layout hands its rows to the next MFMA.
__device__ __forceinline__ int perm_col(int kappa)
{
    return (kappa & ~15) | (((kappa >> 2) & 1) << 3) | (((kappa >> 3) & 1) << 2) | (kappa & 3);
}

// LDS image of one 64-token tile.  X: augmented rows [64][DQK] (content | RIB | zero
// pad | 2 extra columns) plus their transpose [64 rows][64 tokens]; Y: value-like rows
// [64][DVK] (content | zero pad | 2 extra columns) plus the transpose of the first
// 32 columns.  Row strides are padded for conflict-free 16-byte reads.
template <int DQK, int DVK>
struct Lay {
    static constexpr int XS = DQK + 8, YS = DVK + 8;
    static constexpr int XR = 0;
    static constexpr int XT = XR + kT * XS;
    static constexpr int YR = XT + 64 * kTS;
    static constexpr int YT = YR + kT * YS;
    static constexpr int STAGE = YT + 32 * kTS;       // bf16 elements per stage
    static constexpr int KS = DQK / 16, VS = DVK / 16;
    static constexpr int FP = (kT * (DQK / 2) + kNT - 1) / kNT;
};

template <int DQK, int DVK>
struct Regs {
    uint32_t xc[4], yc[4], xf[Lay<DQK, DVK>::FP];
    float e0, e1;
};

// QDO = true : X = Q (scaled by sc | sp), Y = dO, extras = -LSE*log2e and -delta (hi, lo)
// QDO = false: X = K, Y = V, extras = ones
template <int DQK, int DVK, bool QDO>
__device__ __forceinline__ void load_tile(Regs<DQK, DVK> &rg, const Geo &g, int hd, int64_t u, int tile,
                                          const int *tok, const bf16_t *__restrict__ x, int64_t xstride,
                                          const bf16_t *__restrict__ y, int64_t ystride,
                                          const bf16_t *__restrict__ f, const float *__restrict__ lse,
                                          const float *__restrict__ delta)
{
    using L = Lay<DQK, DVK>;
    const int tid = threadIdx.x, pair = tid & 15;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int nl = p * 16 + (tid >> 4);
        int t = tok[tile * kT + nl];
        uint32_t a = 0, b = 0;
        if (t >= 0 && 2 * pair < g.d) {
            a = *(const uint32_t *)(x + (int64_t)t * xstride + hd * g.d + 2 * pair);
            b = *(const uint32_t *)(y + (int64_t)t * ystride + hd * g.d + 2 * pair);
        }
        rg.xc[p] = a;
        rg.yc[p] = b;
    }
    const int n0 = tile * kT;
    const int live = (g.N - n0 < kT ? g.N - n0 : kT) * (g.r >> 1);
    const uint32_t *fsrc = (const uint32_t *)(f + ((int64_t)hd * g.N + n0) * g.r);
#pragma unroll
    for (int p = 0; p < L::FP; ++p) {
        int e = p * kNT + tid;
        rg.xf[p] = (e < live) ? fsrc[e] : 0u;
    }
    rg.e0 = 0.f;
    rg.e1 = 0.f;
    if (QDO && tid < kT && n0 + tid < g.N) {
        rg.e0 = lse[u * g.N + n0 + tid];
        rg.e1 = delta[u * g.N + n0 + tid];
    }
}

template <int DQK, int DVK, bool QDO, bool TRANS_Y>
__device__ __forceinline__ void store_tile(const Regs<DQK, DVK> &rg, const Geo &g, int tile, bf16_t *S, float sc,
                                           float sp, const int *foff, const int *ftoff)
{
    using L = Lay<DQK, DVK>;
    const int tid = threadIdx.x, pair = tid & 15;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        int nl = p * 16 + (tid >> 4);
        if (2 * pair < g.d) {
            uint32_t a = rg.xc[p], b = rg.yc[p];
            if (QDO) a = pack_bf16(lo_bf16(a) * sc, hi_bf16(a) * sc);
            int col = perm_col(nl);
            *(uint32_t *)(S + L::XR + nl * L::XS + 2 * pair) = a;
            S[L::XT + (2 * pair) * kTS + col] = (bf16_t)(a & 0xffffu);
            S[L::XT + (2 * pair + 1) * kTS + col] = (bf16_t)(a >> 16);
            *(uint32_t *)(S + L::YR + nl * L::YS + 2 * pair) = b;
            if (TRANS_Y) {
                S[L::YT + (2 * pair) * kTS + col] = (bf16_t)(b & 0xffffu);
                S[L::YT + (2 * pair + 1) * kTS + col] = (bf16_t)(b >> 16);
            }
        }
    }
    const int fdw = kT * (g.r >> 1);
#pragma unroll
    for (int p = 0; p < L::FP; ++p) {
        int e = p * kNT + tid;
        if (e < fdw) {
            uint32_t a = rg.xf[p];
            if (QDO) a = pack_bf16(lo_bf16(a) * sp, hi_bf16(a) * sp);
            *(uint32_t *)(S + L::XR + foff[p]) = a;
            S[L::XT + ftoff[p]] = (bf16_t)(a & 0xffffu);
            S[L::XT + ftoff[p] + kTS] = (bf16_t)(a >> 16);
        }
    }
    if (tid < kT) {
        const bool valid = tile * kT + tid < g.N;
        uint32_t ex = 0, ey = 0;
        if (valid) {
            if (QDO) {
                ex = split_bf16(-rg.e0 * kLog2e);
                ey = split_bf16(-rg.e1);
            } else {
                ex = 0x3f803f80u;
                ey = 0x3f803f80u;
            }
        }
        *(uint32_t *)(S + L::XR + tid * L::XS + DQK - 2) = ex;
        *(uint32_t *)(S + L::YR + tid * L::YS + DVK - 2) = ey;
    }
}

// Common prologue: XCD-aware block renumbering, token table, LDS clearing, RIB offsets.
template <int DQK, int DVK>
__device__ __forceinline__ void prologue(const Geo &g, int nblk, int64_t &u, int &blk, int &w, int &hd, bf16_t *stages,
                                         int *tok, int *foff, int *ftoff)
{
    using L = Lay<DQK, DVK>;
    const int G = gridDim.x, per = G >> 3, rem = G & 7, xcd = blockIdx.x & 7;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    u = logical / nblk;
    blk = logical - (int)(u * nblk);
    w = (int)(u / g.heads);
    hd = (int)(u - (int64_t)w * g.heads);
    const int tid = threadIdx.x;
    const int ntiles = (g.N + kT - 1) / kT;
    for (int n = tid; n < ntiles * kT; n += kNT) tok[n] = n < g.N ? (int)grid_token(g, w, n) : -1;
    uint32_t *z = (uint32_t *)stages;
    for (int e = tid; e < L::STAGE; e += kNT) z[e] = 0u;        // 2 stages * STAGE bf16 = STAGE dwords
#pragma unroll
    for (int p = 0; p < L::FP; ++p) {
        int e = p * kNT + tid, hr = g.r >> 1;
        int tk = hr > 0 ? e / hr : 0;
        int c = g.d + 2 * (e - tk * hr);
        foff[p] = tk * L::XS + c;
        ftoff[p] = c * kTS + perm_col(tk & 63);
    }
}

template <int N>
__device__ __forceinline__ void read_rows(bf16x8 (&dst)[N], const bf16_t *base, int stride, int row, int hf)
{
#pragma unroll
    for (int t = 0; t < N; ++t) dst[t] = *(const bf16x8 *)(base + row * stride + 16 * t + 8 * hf);
}

__device__ __forceinline__ f32x16 mfma(const bf16x8 &a, const bf16x8 &b, const f32x16 &c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Store one 32-row accumulator block of an augmented gradient: rows are augmented
// columns c = 32*mb + 8*(i/4) + 4*hf + i%4 of this lane's token.
__device__ __forceinline__ void store_aug(const f32x16 &acc, int mb, int hf, const Geo &g, float sc, float sp,
                                          bf16_t *grid_dst, float *part_dst)
{
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
        int c = 32 * mb + 8 * (i >> 2) + 4 * hf + (i & 3);
        if (c < g.d) *(uint32_t *)(grid_dst + c) = pack_bf16(acc[i] * sc, acc[i + 1] * sc);
        else if (c < g.d + g.r) *(float2 *)(part_dst + (c - g.d)) = make_float2(acc[i] * sp, acc[i + 1] * sp);
    }
}

// ---------------------------------------------------------------------------------------
// dQ (+ dF_q partial): queries stationary, keys streamed.
template <int DQK, int DVK>
__global__ __launch_bounds__(kNT, (DQK == 48 && DVK == 32) ? 2 : 1) void mfma_bwd_dq_kernel(Geo g, int nblk, const bf16_t *__restrict__ q,
                                                             const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                                             const bf16_t *__restrict__ fq, const bf16_t *__restrict__ fk,
                                                             const bf16_t *__restrict__ dout,
                                                             const float *__restrict__ lse, const float *__restrict__ delta,
                                                             bf16_t *__restrict__ dq, float *__restrict__ dfq_part)
{
    using L = Lay<DQK, DVK>;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    bf16_t *stage0 = smem, *stage1 = smem + L::STAGE;
    int *tok = (int *)(smem + 2 * L::STAGE);

    int64_t u;
    int blk, w, hd, foff[L::FP], ftoff[L::FP];
    prologue<DQK, DVK>(g, nblk, u, blk, w, hd, smem, tok, foff, ftoff);
    __syncthreads();
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int ntiles = (g.N + kT - 1) / kT;
    const float sc2 = g.scale_c * kLog2e, sp2 = g.scale_p * kLog2e;

    Regs<DQK, DVK> rg;
    bf16x8 Qb[2][L::KS], Gb[2][L::VS];      // stationary B operands: Q_aug' rows, dO_aug rows
    for (int wv = 0; wv < kWaves; ++wv) {
        int qtile = blk * kWaves + wv;
        if (qtile < ntiles) {
            load_tile<DQK, DVK, true>(rg, g, hd, u, qtile, tok, q, g.tstride, dout, (int64_t)g.C, fq, lse, delta);
            store_tile<DQK, DVK, true, false>(rg, g, qtile, stage0, sc2, sp2, foff, ftoff);
        }
        __syncthreads();
        if (wv == wave) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                read_rows<L::KS>(Qb[qb], stage0 + L::XR, L::XS, qb * 32 + col, hf);
                read_rows<L::VS>(Gb[qb], stage0 + L::YR, L::YS, qb * 32 + col, hf);
            }
        }
        __syncthreads();
    }
    const int q0 = (blk * kWaves + wave) * kT;
    if (q0 >= g.N) {        // whole wave past the end: neutral operands (its results are never stored)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
            for (int t = 0; t < L::KS; ++t)
#pragma unroll
                for (int i = 0; i < 8; ++i) Qb[qb][t][i] = (__bf16)0.f;
#pragma unroll
            for (int t = 0; t < L::VS; ++t)
#pragma unroll
                for (int i = 0; i < 8; ++i) Gb[qb][t][i] = (__bf16)0.f;
        }
    }

    f32x16 acc[2][2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[qb][mb][i] = 0.f;

    load_tile<DQK, DVK, false>(rg, g, hd, u, 0, tok, k, g.tstride, v, g.tstride, fk, lse, delta);
    store_tile<DQK, DVK, false, false>(rg, g, 0, stage0, 1.f, 1.f, foff, ftoff);
    __syncthreads();

    for (int tile = 0; tile < ntiles; ++tile) {
        bf16_t *cur = (tile & 1) ? stage1 : stage0, *nxt = (tile & 1) ? stage0 : stage1;
        if (tile + 1 < ntiles)
            load_tile<DQK, DVK, false>(rg, g, hd, u, tile + 1, tok, k, g.tstride, v, g.tstride, fk, lse, delta);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            bf16x8 Ak[L::KS], Av[L::VS], At[2][2];
            read_rows<L::KS>(Ak, cur + L::XR, L::XS, kb * 32 + col, hf);
            read_rows<L::VS>(Av, cur + L::YR, L::YS, kb * 32 + col, hf);
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    At[mb][t] = *(const bf16x8 *)(cur + L::XT + (32 * mb + col) * kTS + kb * 32 + 16 * t + 8 * hf);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                f32x16 S = {0}, D = {0};
#pragma unroll
                for (int t = 0; t < L::KS; ++t) S = mfma(Ak[t], Qb[qb][t], S);     // S^T - LSE (log2 units)
#pragma unroll
                for (int t = 0; t < L::VS; ++t) D = mfma(Av[t], Gb[qb][t], D);     // dP^T - delta
                float ds[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) ds[i] = __builtin_amdgcn_exp2f(S[i]) * D[i];
                bf16x8 B0, B1;
#pragma unroll
                for (int i = 0; i < 8; ++i) { B0[i] = (__bf16)ds[i]; B1[i] = (__bf16)ds[8 + i]; }
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    acc[qb][mb] = mfma(At[mb][0], B0, acc[qb][mb]);
                    acc[qb][mb] = mfma(At[mb][1], B1, acc[qb][mb]);
                }
            }
        }
        if (tile + 1 < ntiles) store_tile<DQK, DVK, false, false>(rg, g, tile + 1, nxt, 1.f, 1.f, foff, ftoff);
        __syncthreads();
    }

#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int n = q0 + qb * 32 + col;
        if (n >= g.N) continue;
        bf16_t *gd = dq + (int64_t)tok[n] * g.C + hd * g.d;
        float *pd = dfq_part + (u * g.N + n) * g.r;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) store_aug(acc[qb][mb], mb, hf, g, g.scale_c, g.scale_p, gd, pd);
    }
}

// ---------------------------------------------------------------------------------------
// dK, dV (+ dF_k partial): keys stationary, queries streamed.
template <int DQK, int DVK>
__global__ __launch_bounds__(kNT, (DQK == 48 && DVK == 32) ? 2 : 1) void mfma_bwd_dkv_kernel(Geo g, int nblk, const bf16_t *__restrict__ q,
                                                              const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                                              const bf16_t *__restrict__ fq, const bf16_t *__restrict__ fk,
                                                              const bf16_t *__restrict__ dout,
                                                              const float *__restrict__ lse, const float *__restrict__ delta,
                                                              bf16_t *__restrict__ dk, bf16_t *__restrict__ dv,
                                                              float *__restrict__ dfk_part)
{
    using L = Lay<DQK, DVK>;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    bf16_t *stage0 = smem, *stage1 = smem + L::STAGE;
    int *tok = (int *)(smem + 2 * L::STAGE);

    int64_t u;
    int blk, w, hd, foff[L::FP], ftoff[L::FP];
    prologue<DQK, DVK>(g, nblk, u, blk, w, hd, smem, tok, foff, ftoff);
    __syncthreads();
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int ntiles = (g.N + kT - 1) / kT;
    const float sc2 = g.scale_c * kLog2e, sp2 = g.scale_p * kLog2e;

    Regs<DQK, DVK> rg;
    bf16x8 Kb[2][L::KS], Vb[2][L::VS];      // stationary B operands: K_aug rows, V_aug rows
    for (int wv = 0; wv < kWaves; ++wv) {
        int ktile = blk * kWaves + wv;
        if (ktile < ntiles) {
            load_tile<DQK, DVK, false>(rg, g, hd, u, ktile, tok, k, g.tstride, v, g.tstride, fk, lse, delta);
            store_tile<DQK, DVK, false, false>(rg, g, ktile, stage0, 1.f, 1.f, foff, ftoff);
        }
        __syncthreads();
        if (wv == wave) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                read_rows<L::KS>(Kb[kb], stage0 + L::XR, L::XS, kb * 32 + col, hf);
                read_rows<L::VS>(Vb[kb], stage0 + L::YR, L::YS, kb * 32 + col, hf);
            }
        }
        __syncthreads();
    }
    const int k0 = (blk * kWaves + wave) * kT;
    if (k0 >= g.N) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int t = 0; t < L::KS; ++t)
#pragma unroll
                for (int i = 0; i < 8; ++i) Kb[kb][t][i] = (__bf16)0.f;
#pragma unroll
            for (int t = 0; t < L::VS; ++t)
#pragma unroll
                for (int i = 0; i < 8; ++i) Vb[kb][t][i] = (__bf16)0.f;
        }
    }

    f32x16 accV[2], accK[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) accV[kb][i] = 0.f;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) accK[kb][mb][i] = 0.f;
    }

    load_tile<DQK, DVK, true>(rg, g, hd, u, 0, tok, q, g.tstride, dout, (int64_t)g.C, fq, lse, delta);
    store_tile<DQK, DVK, true, true>(rg, g, 0, stage0, sc2, sp2, foff, ftoff);
    __syncthreads();

    for (int tile = 0; tile < ntiles; ++tile) {
        bf16_t *cur = (tile & 1) ? stage1 : stage0, *nxt = (tile & 1) ? stage0 : stage1;
        if (tile + 1 < ntiles)
            load_tile<DQK, DVK, true>(rg, g, hd, u, tile + 1, tok, q, g.tstride, dout, (int64_t)g.C, fq, lse, delta);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            bf16x8 Aq[L::KS], Ag[L::VS], Aqt[2][2], Agt[2];
            read_rows<L::KS>(Aq, cur + L::XR, L::XS, qb * 32 + col, hf);
            read_rows<L::VS>(Ag, cur + L::YR, L::YS, qb * 32 + col, hf);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                Agt[t] = *(const bf16x8 *)(cur + L::YT + col * kTS + qb * 32 + 16 * t + 8 * hf);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
                    Aqt[mb][t] = *(const bf16x8 *)(cur + L::XT + (32 * mb + col) * kTS + qb * 32 + 16 * t + 8 * hf);
            }
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x16 S = {0}, D = {0};
#pragma unroll
                for (int t = 0; t < L::KS; ++t) S = mfma(Aq[t], Kb[kb][t], S);     // S - LSE (log2 units)
#pragma unroll
                for (int t = 0; t < L::VS; ++t) D = mfma(Ag[t], Vb[kb][t], D);     // dP - delta
                float p[16], ds[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    p[i] = __builtin_amdgcn_exp2f(S[i]);
                    ds[i] = p[i] * D[i];
                }
                bf16x8 P0, P1, B0, B1;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    P0[i] = (__bf16)p[i];
                    P1[i] = (__bf16)p[8 + i];
                    B0[i] = (__bf16)ds[i];
                    B1[i] = (__bf16)ds[8 + i];
                }
                accV[kb] = mfma(Agt[0], P0, accV[kb]);
                accV[kb] = mfma(Agt[1], P1, accV[kb]);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    accK[kb][mb] = mfma(Aqt[mb][0], B0, accK[kb][mb]);
                    accK[kb][mb] = mfma(Aqt[mb][1], B1, accK[kb][mb]);
                }
            }
        }
        if (tile + 1 < ntiles) store_tile<DQK, DVK, true, true>(rg, g, tile + 1, nxt, sc2, sp2, foff, ftoff);
        __syncthreads();
    }

#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        const int n = k0 + kb * 32 + col;
        if (n >= g.N) continue;
        const int64_t base = (int64_t)tok[n] * g.C + hd * g.d;
        float *pd = dfk_part + (u * g.N + n) * g.r;
        // Q_aug' carries log2(e): undo it here
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) store_aug(accK[kb][mb], mb, hf, g, kLn2, kLn2, dk + base, pd);
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            int c = 8 * (i >> 2) + 4 * hf + (i & 3);
            if (c < g.d) *(uint32_t *)(dv + base + c) = pack_bf16(accV[kb][i], accV[kb][i + 1]);
        }
    }
}

// =======================================================================================
// Fast path (whole 256-token blocks, 32-bit byte offsets, r > 0).  Same mathematics and LDS
// images as the kernels above; what changes is the plumbing around the MFMA loop:
//   - one exposed global-memory latency in the prologue: the first streamed tile and all
//     stationary rows are requested together, and each wave stages its own 64 stationary
//     rows (no workgroup-wide rounds);
//   - streamed tiles are requested two tiles ahead (the loads for tile t+2 are issued at
//     the end of tile t's block and land in LDS at the end of tile t+1's block);
//   - staging has no predicates (idle lanes duplicate a neighbour), builds byte offsets
//     with one 24-bit multiply-add, and writes the transposed images four tokens at a time;
//   - P and dS go to bf16 by truncation (one byte-permute per pair instead of the slow
//     rounding convert); the mean loss of truncation is made up beforehand, as an offset on
//     -LSE*log2(e) (see kTruncLog2);
//   - the dq kernel makes delta = dO.O for its rows while it stages them and writes it out
//     for the dkv kernel, which runs second (no separate pass over O and dO).
// LDS image of one streamed tile of T tokens (same parts as Lay, tile size a parameter).
template <int DQK, int DVK, int T>
struct LayT {
    static constexpr int XS = DQK + 8, YS = DVK + 8, TS = T + 8;
    static constexpr int XR = 0;
    static constexpr int XT = XR + T * XS;
    static constexpr int YR = XT + 64 * TS;
    static constexpr int YT = YR + T * YS;
    static constexpr int EX = YT + 32 * TS;          // 2*T floats: -LSE*log2(e), -delta of the tile's queries
    static constexpr int STAGE = EX + 4 * T;
    static constexpr int KS = DQK / 16, VS = DVK / 16;
};

// P and dS go to bf16 by truncation, which loses half a unit in the last place on average
// (relative 2^-8 * 0.7213 for log-uniform mantissas).  The loss is made up BEFORE the truncation:
// this constant is added to the -LSE * log2(e) that rides with every logit, so P (and with it
// dS = P (dP - delta)) is scaled up by the mean loss and then truncated.  Values that are exactly
// representable (P = 1 of a one-hot row, P = 2^-k of a uniform row) come through unchanged, the
// others are right on average.
constexpr float kTruncLog2 = 0.0040593f;   // log2(1 + 2^-8 * 0.7213)

__device__ __forceinline__ uint32_t trunc_pack(float lo, float hi)
{
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}
__device__ __forceinline__ bf16x8 as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    uint4 w = {a, b, c, d};
    return __builtin_bit_cast(bf16x8, w);
}

template <int DQK, int DVK>
struct FRegs {
    uint32_t xc[4], yc[4], fa[4], fb[DQK == 64 ? 4 : 1];
    float e0, e1;
};

template <int DQK, int DVK, int T>
struct FConst {
    uint32_t lane_c, tsb, dsb;      // channel-pair byte offset in a token; strided / dense token stride in bytes
    uint32_t f_off0, f_off1, frow;  // byte offsets of this lane's RIB dwords; bytes per RIB row
    int tok_idx;                    // first of this lane's 4 tokens in a tile
    int xr, xt, yr, yt, fr0, ft0, fr1, ft1;   // bf16 element offsets inside a stage
};

// Recomputed inside the tile loop from a thread id the optimiser cannot hoist (see
// opaque_tid): a dozen cheap integer instructions per tile instead of a dozen registers
// held across the MFMA block, which is what pushed the dkv kernel into spilling.
__device__ __forceinline__ int opaque_tid()
{
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

template <int DQK, int DVK, int T>
__device__ __forceinline__ FConst<DQK, DVK, T> fconst(const Geo &g, int hd, int tid)
{
    using L = LayT<DQK, DVK, T>;
    constexpr int kTS = L::TS;
    FConst<DQK, DVK, T> c;
    const int grp = tid >> 4, j = tid & 15;
    const int hp = g.d >> 1, rh = g.r >> 1;
    const int pair = j < hp ? j : hp - 1;
    const int f0 = j < rh ? j : rh - 1, f1 = 16 + j < rh ? 16 + j : rh - 1;
    const int pc = perm_col(grp * 4);
    c.lane_c = (uint32_t)(hd * g.d + 2 * pair) * 2u;
    c.tsb = (uint32_t)g.tstride * 2u;
    c.dsb = (uint32_t)g.C * 2u;
    c.f_off0 = (uint32_t)f0 * 4u;
    c.f_off1 = (uint32_t)f1 * 4u;
    c.frow = (uint32_t)g.r * 2u;
    c.tok_idx = grp * 4;
    c.xr = L::XR + grp * 4 * L::XS + 2 * pair;
    c.xt = L::XT + (2 * pair) * kTS + pc;
    c.yr = L::YR + grp * 4 * L::YS + 2 * pair;
    c.yt = L::YT + (2 * pair) * kTS + pc;
    c.fr0 = L::XR + grp * 4 * L::XS + g.d + 2 * f0;
    c.ft0 = L::XT + (g.d + 2 * f0) * kTS + pc;
    c.fr1 = L::XR + grp * 4 * L::XS + g.d + 2 * f1;
    c.ft1 = L::XT + (g.d + 2 * f1) * kTS + pc;
    return c;
}

// Request tile `tile` of the streamed operand pair.  QDO: X = q (strided), Y = dO (dense),
// extras = LSE, delta.  Otherwise X = k, Y = v (both strided).
template <int DQK, int DVK, int T, bool QDO>
__device__ __forceinline__ void fload(FRegs<DQK, DVK> &rg, const FConst<DQK, DVK, T> &c, const Geo &g, int64_t u, int tile,
                                      const TokMap &tok, const char *xb, const char *yb, const char *fbase,
                                      const float *__restrict__ lse, const float *__restrict__ delta)
{
    constexpr int kT = T;
    const char *fb = fbase + (uint32_t)tile * (uint32_t)kT * c.frow;
    int tq[4];
    tok.quad(tile * kT + c.tok_idx, tq);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t t = (uint32_t)tq[p];
        rg.xc[p] = *(const uint32_t *)(xb + (__umul24(t, c.tsb) + c.lane_c));
        rg.yc[p] = *(const uint32_t *)(yb + (__umul24(t, QDO ? c.dsb : c.tsb) + c.lane_c));
        const uint32_t row = (uint32_t)(c.tok_idx + p) * c.frow;
        rg.fa[p] = *(const uint32_t *)(fb + row + c.f_off0);
        if (DQK == 64) rg.fb[p] = *(const uint32_t *)(fb + row + c.f_off1);
    }
    if (QDO && threadIdx.x < kT) {
        rg.e0 = lse[u * g.N + tile * kT + threadIdx.x];
        rg.e1 = delta[u * g.N + tile * kT + threadIdx.x];
    }
}

// four dwords (tokens t..t+3, one channel pair) -> the two transposed rows, 8 bytes each
template <int kTS>
__device__ __forceinline__ void store_t4(bf16_t *dst, const uint32_t (&w)[4])
{
    uint2 even, odd;
    even.x = __builtin_amdgcn_perm(w[1], w[0], 0x05040100u);
    even.y = __builtin_amdgcn_perm(w[3], w[2], 0x05040100u);
    odd.x = __builtin_amdgcn_perm(w[1], w[0], 0x07060302u);
    odd.y = __builtin_amdgcn_perm(w[3], w[2], 0x07060302u);
    *(uint2 *)dst = even;
    *(uint2 *)(dst + kTS) = odd;
}

template <int DQK, int DVK, int T, bool QDO, bool TRANS_Y, bool SCALE, bool XC>
__device__ __forceinline__ void fstore(const FRegs<DQK, DVK> &rg, const FConst<DQK, DVK, T> &c, bf16_t *S, float sc, float sp)
{
    using L = LayT<DQK, DVK, T>;
    constexpr int kT = T, kTS = L::TS;
    uint32_t x[4], fa[4], fb[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        x[p] = rg.xc[p];
        fa[p] = rg.fa[p];
        fb[p] = DQK == 64 ? rg.fb[p] : 0u;
        if (SCALE) {
            x[p] = pack_bf16(lo_bf16(x[p]) * sc, hi_bf16(x[p]) * sc);
            fa[p] = pack_bf16(lo_bf16(fa[p]) * sp, hi_bf16(fa[p]) * sp);
            if (DQK == 64) fb[p] = pack_bf16(lo_bf16(fb[p]) * sp, hi_bf16(fb[p]) * sp);
        }
        *(uint32_t *)(S + c.xr + p * L::XS) = x[p];
        *(uint32_t *)(S + c.yr + p * L::YS) = rg.yc[p];
        *(uint32_t *)(S + c.fr0 + p * L::XS) = fa[p];
        if (DQK == 64) *(uint32_t *)(S + c.fr1 + p * L::XS) = fb[p];
    }
    store_t4<kTS>(S + c.xt, x);
    store_t4<kTS>(S + c.ft0, fa);
    if (DQK == 64) store_t4<kTS>(S + c.ft1, fb);
    if (TRANS_Y) store_t4<kTS>(S + c.yt, rg.yc);
    if (XC) {
        if (QDO && threadIdx.x < kT) {
            float *ex = (float *)(S + L::EX);
            ex[threadIdx.x] = kTruncLog2 - rg.e0 * kLog2e;
            ex[kT + threadIdx.x] = -rg.e1;
        }
    } else if (threadIdx.x < kT) {
        uint32_t ex = 0x3f803f80u, ey = 0x3f803f80u;
        if (QDO) {
            ex = split_bf16(kTruncLog2 - rg.e0 * kLog2e);
            ey = split_bf16(-rg.e1);
        }
        *(uint32_t *)(S + L::XR + threadIdx.x * L::XS + DQK - 2) = ex;
        *(uint32_t *)(S + L::YR + threadIdx.x * L::YS + DVK - 2) = ey;
    }
}

// Zero the columns of one augmented row pair that no staging code writes: [d+r, DQK) of the X row and
// [d, DVK) of the Y row, minus the two columns that carry LSE / delta when those ride in columns.
template <int DQK, int DVK, bool XC>
__device__ __forceinline__ void clear_pad_columns(const Geo &g, bf16_t *xrow, bf16_t *yrow)
{
    for (int c = g.d + g.r; c < DQK - (XC ? 0 : 2); c += 2) *(uint32_t *)(xrow + c) = 0u;
    for (int c = g.d; c < DVK - (XC ? 0 : 2); c += 2) *(uint32_t *)(yrow + c) = 0u;
}

// Each wave stages its own 64 stationary rows (X rows [64][XS], Y rows [64][YS], extras
// included) into its private LDS area `W` and reads them back as MFMA B operands.
//
// MAKE_DELTA (QDO only): the rows' delta_i = dO_i . O_i (paper Sec. 2.2 backward; the softmax Jacobian's row
// term) is formed here from the dO words the lanes hold anyway plus the matching O words, instead of
// being read: 16 lanes share a token, each multiplies its channel pair, four DPP steps add the 16
// partial sums, and a lane permute hands row `lane` its value.  The values are also written to
// `delta_out` for the dkv kernel, which streams these rows later.  `e1_out` returns the lane's delta.
// `from_o` false (uniform): an earlier pass has made delta already (the gated backward's pass over dO', G, O)
// and it is read instead.
template <int DQK, int DVK, bool QDO, bool SCALE, bool XC, bool MAKE_DELTA = false>
__device__ __forceinline__ void stationary_rows(const Geo &g, int hd, int64_t u, int n0, const TokMap &tok, const char *xb,
                                                const char *yb, const bf16_t *f, const float *__restrict__ lse,
                                                const float *__restrict__ delta, float sc, float sp, bf16_t *W,
                                                bf16x8 (&Xb)[2][DQK / 16], bf16x8 (&Yb)[2][DVK / 16],
                                                const char *ob = nullptr, float *__restrict__ delta_out = nullptr,
                                                float *e1_out = nullptr, bool from_o = true)
{
    using L = Lay<DQK, DVK>;
    const int lane = threadIdx.x & 63, sub = lane >> 4, j = lane & 15, col = lane & 31, hf = lane >> 5;
    const int hp = g.d >> 1, rh = g.r >> 1;
    const int pair = j < hp ? j : hp - 1;
    const int f0 = j < rh ? j : rh - 1, f1 = 16 + j < rh ? 16 + j : rh - 1;
    const uint32_t lane_c = (uint32_t)(hd * g.d + 2 * pair) * 2u;
    const uint32_t tsb = (uint32_t)g.tstride * 2u, ysb = QDO ? (uint32_t)g.C * 2u : tsb, frow = (uint32_t)g.r * 2u;
    const char *fb = (const char *)(f + ((int64_t)hd * g.N + n0) * g.r);
    bf16_t *Xs = W, *Ys = W + kT * L::XS;
    uint32_t xx[16], yy[16], fa[16], fb2[DQK == 64 ? 16 : 1], oo[MAKE_DELTA ? 16 : 1];
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        const int row = p * 4 + sub;
        const uint32_t t = (uint32_t)tok[n0 + row];
        xx[p] = *(const uint32_t *)(xb + (__umul24(t, tsb) + lane_c));
        yy[p] = *(const uint32_t *)(yb + (__umul24(t, ysb) + lane_c));
        if (MAKE_DELTA && from_o) oo[p] = *(const uint32_t *)(ob + (__umul24(t, ysb) + lane_c));
        fa[p] = *(const uint32_t *)(fb + (uint32_t)row * frow + 4 * f0);
        if (DQK == 64) fb2[p] = *(const uint32_t *)(fb + (uint32_t)row * frow + 4 * f1);
    }
    float e0 = 0.f, e1 = 0.f;
    if (QDO && !XC) e0 = lse[u * g.N + n0 + lane];
    if (QDO && ((!MAKE_DELTA && !XC) || (MAKE_DELTA && !from_o))) e1 = delta[u * g.N + n0 + lane];   // (made by an earlier pass)
    if (MAKE_DELTA && !from_o && e1_out) *e1_out = e1;
    if (MAKE_DELTA && from_o) {
        // part[p]: this lane's channel pair of row p*4+sub (lanes past the last pair hold a copy of it and
        // contribute nothing).  The 16 lanes of a group then reduce and scatter in four halving steps:
        // a lane keeps the rows whose index bit matches its own lane bit and adds what its partner
        // (lane ^ 15, ^ 7, ^ 2, ^ 1: all DPP patterns) held for them, so lane j ends with row j*4+sub.
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        float part[16];
#pragma unroll
        for (int p = 0; p < 16; ++p)
            part[p] = j < hp ? __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, yy[p]), __builtin_bit_cast(bf16x2, oo[p]),
                                                               0.f, false)
                             : 0.f;
#define RIB_DPP(x, ctrl) __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (x)), (ctrl), 0xF, 0xF, true))
        const bool b3 = (j & 8) != 0, b2 = (j & 4) != 0, b1 = (j & 2) != 0, b0 = (j & 1) != 0;
        float h8[8], h4[4], h2[2];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float keep = b3 ? part[8 + i] : part[i], give = b3 ? part[i] : part[8 + i];
            h8[i] = keep + RIB_DPP(give, 0x140);        // row_mirror: lane ^ 15
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float keep = b2 ? h8[4 + i] : h8[i], give = b2 ? h8[i] : h8[4 + i];
            h4[i] = keep + RIB_DPP(give, 0x141);        // row_half_mirror: lane ^ 7
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const float keep = b1 ? h4[2 + i] : h4[i], give = b1 ? h4[i] : h4[2 + i];
            h2[i] = keep + RIB_DPP(give, 0x4E);         // quad_perm [2,3,0,1]: lane ^ 2
        }
        const float keep = b0 ? h2[1] : h2[0], give = b0 ? h2[0] : h2[1];
        const float mine = keep + RIB_DPP(give, 0xB1);  // quad_perm [1,0,3,2]: lane ^ 1
#undef RIB_DPP
        // row `lane` sits in lane (lane & 3) * 16 + (lane >> 2)
        e1 = __shfl(mine, (lane & 3) * 16 + (lane >> 2));
        delta_out[u * g.N + n0 + lane] = e1;
        if (e1_out) *e1_out = e1;
    }
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        const int row = p * 4 + sub;
        uint32_t a = xx[p], b = fa[p], b2 = DQK == 64 ? fb2[p] : 0u;
        if (SCALE) {
            a = pack_bf16(lo_bf16(a) * sc, hi_bf16(a) * sc);
            b = pack_bf16(lo_bf16(b) * sp, hi_bf16(b) * sp);
            if (DQK == 64) b2 = pack_bf16(lo_bf16(b2) * sp, hi_bf16(b2) * sp);
        }
        *(uint32_t *)(Xs + row * L::XS + 2 * pair) = a;
        *(uint32_t *)(Xs + row * L::XS + g.d + 2 * f0) = b;
        if (DQK == 64) *(uint32_t *)(Xs + row * L::XS + g.d + 2 * f1) = b2;
        *(uint32_t *)(Ys + row * L::YS + 2 * pair) = yy[p];
    }
    if (!XC) {
        uint32_t ex = 0x3f803f80u, ey = 0x3f803f80u;
        if (QDO) {
            ex = split_bf16(kTruncLog2 - e0 * kLog2e);
            ey = split_bf16(-e1);
        }
        *(uint32_t *)(Xs + lane * L::XS + DQK - 2) = ex;
        *(uint32_t *)(Ys + lane * L::YS + DVK - 2) = ey;
    }
    // the padding columns of the stationary operands must read zero: whatever a streamed tile
    // holds in the same columns is then multiplied away
    clear_pad_columns<DQK, DVK, XC>(g, Xs + lane * L::XS, Ys + lane * L::YS);
    __syncthreads();
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        read_rows<DQK / 16>(Xb[b], Xs, L::XS, b * 32 + col, hf);
        read_rows<DVK / 16>(Yb[b], Ys, L::YS, b * 32 + col, hf);
    }
    __syncthreads();
}

// ---- epilogue through LDS: the accumulator layout gives a lane 16 rows of ONE token, and
// storing from there would touch 32 token rows per instruction.  Each wave parks the fp32
// accumulators of its 64 tokens in a private LDS area (rows of kARS floats: the odd stride keeps
// the column-wise writes conflict-free) without any per-element decision, and writes them out
// with 16 lanes per token, scaling and rounding on the way.  The area is private to the wave and
// the LDS serves a wave's instructions in order, so no workgroup barrier is needed around it.
constexpr int kARS = 65;
constexpr int kWaveOut = 64 * kARS * 4;      // bytes per wave

// one 32 x 32 accumulator block: this lane's token row, columns 32*mb + ...
__device__ __forceinline__ void stash_block(const f32x16 &acc, int mb, int hf, float *arow)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) arow[32 * mb + 8 * (i >> 2) + 4 * hf + (i & 3)] = acc[i];
}

// Byte offsets, in a dense [tokens][C] grid tensor, of the channel pair this lane stores for each of its 16
// rows (rows p*4 + sub of the wave's 64, pair j of head hd).  They fit 32 bits on this path.
__device__ __forceinline__ void row_offsets(uint32_t (&off)[16], const TokMap &tok, int n0, int hd, const Geo &g)
{
    const int lane = threadIdx.x & 63, sub = lane >> 4, j = lane & 15;
    const uint32_t chan = (uint32_t)(hd * g.d + 2 * j) * 2u, row_bytes = (uint32_t)g.C * 2u;
#pragma unroll
    for (int p = 0; p < 16; ++p) off[p] = (uint32_t)tok[n0 + p * 4 + sub] * row_bytes + chan;
}

// columns [0, d) of the wave's 64 rows -> a grid tensor (bf16), times `scale`
__device__ __forceinline__ void flush_rows(const float *As, float scale, bf16_t *__restrict__ dst, const uint32_t (&off)[16],
                                           const Geo &g)
{
    const int lane = threadIdx.x & 63, sub = lane >> 4, j = lane & 15;
    if (2 * j < g.d) {
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = p * 4 + sub;
            const float a = As[row * kARS + 2 * j] * scale, b = As[row * kARS + 2 * j + 1] * scale;
            *(uint32_t *)((char *)dst + off[p]) = pack_bf16(a, b);
        }
    }
}

// columns [d, d+r) of the wave's 64 rows -> this unit's RIB partial (contiguous in memory), times `scale`.
// 16 columns per pass; the branches on r are uniform, only a rank under 16 needs a lane predicate.
__device__ __forceinline__ void flush_partial(const float *As, float scale, float *__restrict__ part, const Geo &g)
{
    const int lane = threadIdx.x & 63, sub = lane >> 4, j = lane & 15, r = g.r;
    const float *Fs = As + g.d;
    for (int c0 = 0; c0 < r; c0 += 16) {
        const bool whole = c0 + 16 <= r;
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = p * 4 + sub;
            if (whole || c0 + j < r) part[row * r + c0 + j] = Fs[row * kARS + c0 + j] * scale;
        }
    }
}

template <int DQK, int DVK, int T, int WAVES>
struct FSmem {
    using L = LayT<DQK, DVK, T>;
    static constexpr int STAT = WAVES * (64 * L::XS + 64 * L::YS);             // stationary staging, bf16
    static constexpr int OUTB = WAVES * kWaveOut / 2;                            // epilogue staging, bf16 units
    static constexpr int ELEMS0 = (2 * L::STAGE > STAT ? 2 * L::STAGE : STAT);
    static constexpr int ELEMS = (ELEMS0 > OUTB ? ELEMS0 : OUTB);
    static constexpr int ELEMS16 = (ELEMS + 7) / 8 * 8;
    static constexpr size_t BYTES = (size_t)ELEMS16 * sizeof(bf16_t);
};

// padding columns of the row images of both stages (see clear_pad_columns)
template <int DQK, int DVK, int T, int NT, bool XC>
__device__ __forceinline__ void clear_stage_pads(const Geo &g, bf16_t *stage0, bf16_t *stage1)
{
    using L = LayT<DQK, DVK, T>;
    for (int e = threadIdx.x; e < 2 * T; e += NT) {
        bf16_t *st = e < T ? stage0 : stage1;
        const int row = e < T ? e : e - T;
        clear_pad_columns<DQK, DVK, XC>(g, st + L::XR + row * L::XS, st + L::YR + row * L::YS);
    }
}

__device__ __forceinline__ void block_coords(const Geo &g, int nblk, int64_t &u, int &blk, int &w, int &hd)
{
    const int G = gridDim.x, per = G >> 3, rem = G & 7, xcd = blockIdx.x & 7;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    u = logical / nblk;
    blk = logical - (int)(u * nblk);
    w = (int)(u / g.heads);
    hd = (int)(u - (int64_t)w * g.heads);
}

// dQ (+ dF_q partial), fast path.
template <int DQK, int DVK, int T, int WAVES, bool XC>
__global__ __launch_bounds__(WAVES * 64, (DVK == 32) ? 2 : 1) void mfma_bwd_dq_fast_kernel(
    Geo g, int nblk, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const bf16_t *__restrict__ fq, const bf16_t *__restrict__ fk, const bf16_t *__restrict__ out,
    const bf16_t *__restrict__ dout, const float *__restrict__ lse, float *__restrict__ delta, bf16_t *__restrict__ dq,
    float *__restrict__ dfq_part)
{
    using L = LayT<DQK, DVK, T>;
    using Sm = FSmem<DQK, DVK, T, WAVES>;
    constexpr int kT = T, kTS = L::TS, kWaves = WAVES, kNT = WAVES * 64, NB = T / 32;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    bf16_t *stage0 = smem, *stage1 = smem + L::STAGE;

    int64_t u;
    int blk, w, hd;
    block_coords(g, nblk, u, blk, w, hd);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int ntiles = g.N / kT;
    const float sc2 = g.scale_c * kLog2e, sp2 = g.scale_p * kLog2e;

    const TokMap tok = fill_tok_map<kNT>(g, w, (int *)(smem + Sm::ELEMS16));
    __syncthreads();

    const FConst<DQK, DVK, T> c = fconst<DQK, DVK, T>(g, hd, threadIdx.x);
    const char *kb = (const char *)k, *vb = (const char *)v;
    const char *fkb = (const char *)(fk + (int64_t)hd * g.N * g.r);
    FRegs<DQK, DVK> rg;
    fload<DQK, DVK, T, false>(rg, c, g, u, 0, tok, kb, vb, fkb, lse, delta);

    const int q0 = (blk * kWaves + wave) * 64;
    bf16x8 Qb[2][L::KS], Gb[2][L::VS];
    // (this kernel also makes delta = dO . O for its rows and leaves it in `delta` for the dkv kernel,
    // which therefore runs after it; a gated call has it from its pass over dO', G and O already)
    float my_delta = 0.f;
    stationary_rows<DQK, DVK, true, true, XC, true>(g, hd, u, q0, tok, (const char *)q, (const char *)dout, fq, lse, delta, sc2,
                                                    sp2, smem + wave * (64 * L::XS + 64 * L::YS), Qb, Gb, (const char *)out,
                                                    delta, &my_delta, g.gate == nullptr);
    // LDS is not cleared wholesale.  The padding columns of the streamed row images only ever
    // multiply the zero padding of the stationary operands, but they must be finite for that:
    // they are zeroed once here, in both stages (nothing writes them afterwards).  Unwritten rows
    // of the transposed images only feed accumulator rows that are never stored.
    clear_stage_pads<DQK, DVK, T, kNT, XC>(g, stage0, stage1);
    fstore<DQK, DVK, T, false, false, false, XC>(rg, c, stage0, 1.f, 1.f);
    fload<DQK, DVK, T, false>(rg, c, g, u, ntiles > 1 ? 1 : 0, tok, kb, vb, fkb, lse, delta);
    __syncthreads();

    f32x16 acc[2][2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[qb][mb][i] = 0.f;
    // XC: a lane owns one query per block, so -LSE*log2(e) and -delta are two lane constants
    // added to the finished scores.
    float nl[2] = {0.f, 0.f}, nd[2] = {0.f, 0.f};
    if (XC) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            nl[qb] = kTruncLog2 - lse[u * g.N + q0 + qb * 32 + col] * kLog2e;
            nd[qb] = -__shfl(my_delta, qb * 32 + col);
        }
    }

    for (int tile = 0; tile < ntiles; ++tile) {
        bf16_t *cur = (tile & 1) ? stage1 : stage0, *nxt = (tile & 1) ? stage0 : stage1;
#pragma unroll
        for (int kb2 = 0; kb2 < NB; ++kb2) {
            bf16x8 Ak[L::KS], Av[L::VS], At[2][2];
            read_rows<L::KS>(Ak, cur + L::XR, L::XS, kb2 * 32 + col, hf);
            read_rows<L::VS>(Av, cur + L::YR, L::YS, kb2 * 32 + col, hf);
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    At[mb][t] = *(const bf16x8 *)(cur + L::XT + (32 * mb + col) * kTS + kb2 * 32 + 16 * t + 8 * hf);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                f32x16 S = {0}, D = {0};
#pragma unroll
                for (int t = 0; t < L::KS; ++t) S = mfma(Ak[t], Qb[qb][t], S);
#pragma unroll
                for (int t = 0; t < L::VS; ++t) D = mfma(Av[t], Gb[qb][t], D);
                uint32_t wds[8];
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    if (XC)
                        wds[i >> 1] = trunc_pack(__builtin_amdgcn_exp2f(S[i] + nl[qb]) * (D[i] + nd[qb]),
                                                 __builtin_amdgcn_exp2f(S[i + 1] + nl[qb]) * (D[i + 1] + nd[qb]));
                    else
                        wds[i >> 1] = trunc_pack(__builtin_amdgcn_exp2f(S[i]) * D[i],
                                                 __builtin_amdgcn_exp2f(S[i + 1]) * D[i + 1]);
                }
                const bf16x8 B0 = as_bf16x8(wds[0], wds[1], wds[2], wds[3]);
                const bf16x8 B1 = as_bf16x8(wds[4], wds[5], wds[6], wds[7]);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    acc[qb][mb] = mfma(At[mb][0], B0, acc[qb][mb]);
                    acc[qb][mb] = mfma(At[mb][1], B1, acc[qb][mb]);
                }
            }
        }
        fstore<DQK, DVK, T, false, false, false, XC>(rg, c, nxt, 1.f, 1.f);
        fload<DQK, DVK, T, false>(rg, c, g, u, tile + 2 < ntiles ? tile + 2 : ntiles - 1, tok, kb, vb, fkb, lse, delta);
        __syncthreads();
    }

    // (the loop's last barrier has passed: the tiles are free)
    float *As = (float *)((char *)smem + wave * kWaveOut);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) stash_block(acc[qb][mb], mb, hf, As + (qb * 32 + col) * kARS);
    __builtin_amdgcn_wave_barrier();
    uint32_t roff[16];
    row_offsets(roff, tok, q0, hd, g);
    flush_rows(As, g.scale_c, dq, roff, g);
    flush_partial(As, g.scale_p, dfq_part + (u * g.N + q0) * g.r, g);
}

// dK, dV (+ dF_k partial), fast path.
template <int DQK, int DVK, int T, int WAVES, bool XC>
__global__ __launch_bounds__(WAVES * 64, (DVK == 32) ? 2 : 1) void mfma_bwd_dkv_fast_kernel(
    Geo g, int nblk, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
    const bf16_t *__restrict__ fq, const bf16_t *__restrict__ fk, const bf16_t *__restrict__ dout,
    const float *__restrict__ lse, const float *__restrict__ delta, bf16_t *__restrict__ dk, bf16_t *__restrict__ dv,
    float *__restrict__ dfk_part)
{
    using L = LayT<DQK, DVK, T>;
    using Sm = FSmem<DQK, DVK, T, WAVES>;
    constexpr int kT = T, kTS = L::TS, kWaves = WAVES, kNT = WAVES * 64, NB = T / 32;
    extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
    bf16_t *stage0 = smem, *stage1 = smem + L::STAGE;

    int64_t u;
    int blk, w, hd;
    block_coords(g, nblk, u, blk, w, hd);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;
    const int ntiles = g.N / kT;
    const float sc2 = g.scale_c * kLog2e, sp2 = g.scale_p * kLog2e;

    const TokMap tok = fill_tok_map<kNT>(g, w, (int *)(smem + Sm::ELEMS16));
    __syncthreads();

    const FConst<DQK, DVK, T> c = fconst<DQK, DVK, T>(g, hd, threadIdx.x);
    const char *qb_ = (const char *)q, *gb_ = (const char *)dout;
    const char *fqb = (const char *)(fq + (int64_t)hd * g.N * g.r);
    FRegs<DQK, DVK> rg;
    fload<DQK, DVK, T, true>(rg, c, g, u, 0, tok, qb_, gb_, fqb, lse, delta);

    const int k0 = (blk * kWaves + wave) * 64;
    bf16x8 Kb[2][L::KS], Vb[2][L::VS];
    // The logits must be the forward's bit for bit, or P = exp2(S - LSE) is off by the difference of
    // two roundings (for logits of size 100 that is a factor, not a rounding error): Q_aug is scaled
    // and rounded exactly as the forward and the dq kernel do it -- here on the streamed side, a few
    // vector instructions per tile -- and K_aug enters as it is.
    stationary_rows<DQK, DVK, false, false, XC>(g, hd, u, k0, tok, (const char *)k, (const char *)v, fk, lse, delta, 1.f, 1.f,
                                      smem + wave * (64 * L::XS + 64 * L::YS), Kb, Vb);
    clear_stage_pads<DQK, DVK, T, kNT, XC>(g, stage0, stage1);
    fstore<DQK, DVK, T, true, true, true, XC>(rg, c, stage0, sc2, sp2);
    fload<DQK, DVK, T, true>(rg, c, g, u, ntiles > 1 ? 1 : 0, tok, qb_, gb_, fqb, lse, delta);
    __syncthreads();

    f32x16 accV[2], accK[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) accV[kb][i] = 0.f;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) accK[kb][mb][i] = 0.f;
    }

    for (int tile = 0; tile < ntiles; ++tile) {
        bf16_t *cur = (tile & 1) ? stage1 : stage0, *nxt = (tile & 1) ? stage0 : stage1;
#pragma unroll
        for (int qb = 0; qb < NB; ++qb) {
            // With 64 augmented columns the registers are short: the transposed operands are then
            // read per key block, right where they are used, instead of once per query block.
            constexpr bool kLate = DQK == 64;
            bf16x8 Aq[L::KS], Ag[L::VS], Aqt[2][2], Agt[2];
            read_rows<L::KS>(Aq, cur + L::XR, L::XS, qb * 32 + col, hf);
            read_rows<L::VS>(Ag, cur + L::YR, L::YS, qb * 32 + col, hf);
            if (!kLate) {
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    Agt[t] = *(const bf16x8 *)(cur + L::YT + col * kTS + qb * 32 + 16 * t + 8 * hf);
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
                        Aqt[mb][t] = *(const bf16x8 *)(cur + L::XT + (32 * mb + col) * kTS + qb * 32 + 16 * t + 8 * hf);
                }
            }
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                f32x16 S = {0}, D = {0};
                if (XC) {
                    // accumulator row 8j + 4*hf + e is query qb*32 + that: four consecutive floats per j
                    // (offset made opaque so that the reads are repeated per key block instead of
                    // being kept in 32 registers across both)
                    int exo = qb * 32 + 4 * hf;
                    asm volatile("" : "+v"(exo));
                    const float *ex = (const float *)(cur + L::EX) + exo;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float4 a = *(const float4 *)(ex + 8 * j), b = *(const float4 *)(ex + kT + 8 * j);
                        S[4 * j] = a.x, S[4 * j + 1] = a.y, S[4 * j + 2] = a.z, S[4 * j + 3] = a.w;
                        D[4 * j] = b.x, D[4 * j + 1] = b.y, D[4 * j + 2] = b.z, D[4 * j + 3] = b.w;
                    }
                }
#pragma unroll
                for (int t = 0; t < L::KS; ++t) S = mfma(Aq[t], Kb[kb][t], S);
#pragma unroll
                for (int t = 0; t < L::VS; ++t) D = mfma(Ag[t], Vb[kb][t], D);
                uint32_t wp[8], wds[8];
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(S[i]), p1 = __builtin_amdgcn_exp2f(S[i + 1]);
                    wp[i >> 1] = trunc_pack(p0, p1);
                    wds[i >> 1] = trunc_pack(p0 * D[i], p1 * D[i + 1]);
                }
                if (kLate) {
                    int to = qb * 32 + 8 * hf + col * kTS;
                    asm volatile("" : "+v"(to));
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        Agt[t] = *(const bf16x8 *)(cur + L::YT + to + 16 * t);
#pragma unroll
                        for (int mb = 0; mb < 2; ++mb)
                            Aqt[mb][t] = *(const bf16x8 *)(cur + L::XT + 32 * mb * kTS + to + 16 * t);
                    }
                }
                accV[kb] = mfma(Agt[0], as_bf16x8(wp[0], wp[1], wp[2], wp[3]), accV[kb]);
                accV[kb] = mfma(Agt[1], as_bf16x8(wp[4], wp[5], wp[6], wp[7]), accV[kb]);
                const bf16x8 B0 = as_bf16x8(wds[0], wds[1], wds[2], wds[3]);
                const bf16x8 B1 = as_bf16x8(wds[4], wds[5], wds[6], wds[7]);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb) {
                    accK[kb][mb] = mfma(Aqt[mb][0], B0, accK[kb][mb]);
                    accK[kb][mb] = mfma(Aqt[mb][1], B1, accK[kb][mb]);
                }
            }
        }
        {
            const FConst<DQK, DVK, T> cc = fconst<DQK, DVK, T>(g, hd, opaque_tid());
            fstore<DQK, DVK, T, true, true, true, XC>(rg, cc, nxt, sc2, sp2);
            fload<DQK, DVK, T, true>(rg, cc, g, u, tile + 2 < ntiles ? tile + 2 : ntiles - 1, tok, qb_, gb_, fqb, lse,
                                     delta);
        }
        __syncthreads();
    }

    float *As = (float *)((char *)smem + wave * kWaveOut);
    // dK and the dF_k partial first, then dV through the same area
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) stash_block(accK[kb][mb], mb, hf, As + (kb * 32 + col) * kARS);
    __builtin_amdgcn_wave_barrier();
    // (the streamed Q_aug rows carry scale * log2 e: undo the log2 e here)
    uint32_t roff[16];
    row_offsets(roff, tok, k0, hd, g);
    flush_rows(As, kLn2, dk, roff, g);
    flush_partial(As, kLn2, dfk_part + (u * g.N + k0) * g.r, g);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) stash_block(accV[kb], 0, hf, As + (kb * 32 + col) * kARS);
    __builtin_amdgcn_wave_barrier();
    flush_rows(As, 1.f, dv, roff, g);
}

static bool bwd_fast_ok(const Geo &g)
{
    const int64_t tokens = (int64_t)g.B * g.H * g.W;
    return g.r > 0 && g.r <= 34 && g.N % 256 == 0 && tokens < (1 << 24) && g.tstride * 2 < (1 << 24) &&
           tokens * g.tstride * 2 < ((int64_t)1 << 32);
}

// Launch the fast pair with workgroups of WAVES waves and streamed tiles of T tokens.
template <int DQK, int DVK, int T, int WAVES, bool XC>
hipError_t launch_fast(const Geo &g, const void *q, const void *k, const void *v, const void *fq, const void *fk,
                       const void *out, const void *dout, const float *lse, float *delta, void *dq, void *dk, void *dv,
                       float *pq, float *pk, hipStream_t st)
{
    const size_t smem = FSmem<DQK, DVK, T, WAVES>::BYTES + (size_t)2 * g.M * sizeof(int);
    if (smem > (size_t)kMaxDynLds) return hipErrorInvalidValue;
    auto kdkv = mfma_bwd_dkv_fast_kernel<DQK, DVK, T, WAVES, XC>;
    auto kdq = mfma_bwd_dq_fast_kernel<DQK, DVK, T, WAVES, XC>;
    hipError_t pe = prepare_kernel((const void *)kdkv, nullptr);
    if (pe == hipSuccess) pe = prepare_kernel((const void *)kdq, nullptr);
    if (pe != hipSuccess) return pe;
    const int nblk = g.N / (WAVES * 64);
    const dim3 grid((unsigned)(g.units * nblk)), block(WAVES * 64);
    // dq first: it writes the delta rows the dkv kernel streams
    hipLaunchKernelGGL(kdq, grid, block, smem, st, g, nblk, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                       (const bf16_t *)fq, (const bf16_t *)fk, (const bf16_t *)out, (const bf16_t *)dout, lse, delta,
                       (bf16_t *)dq, pq);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kdkv, grid, block, smem, st, g, nblk, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                       (const bf16_t *)fq, (const bf16_t *)fk, (const bf16_t *)dout, lse, (const float *)delta,
                       (bf16_t *)dk, (bf16_t *)dv, pk);
    return hipGetLastError();
}

template <int DQK, int DVK, bool XC = false>
hipError_t launch(const Geo &g, const void *q, const void *k, const void *v, const void *fq, const void *fk,
                  const void *out, const void *dout, const float *lse, void *dq, void *dk, void *dv, float *dfq,
                  float *dfk, void *ws, hipStream_t st)
{
    using L = Lay<DQK, DVK>;
    const BwdWs l = bwd_ws_layout(g);
    float *delta = (float *)((char *)ws + l.delta_off);
    float *pq = (float *)((char *)ws + l.dfq_off);
    float *pk = (float *)((char *)ws + l.dfk_off);
    hipError_t e = hipSuccess;
    if (bwd_fast_ok(g)) {
        // (delta is made inside the dq kernel; for a gated call the caller's pass over dO', G, O has
        // written the same values already)
        // Large windows with enough workgroups to go round: 8 waves share each streamed tile (128
        // tokens), which halves the staging work per wave (measured +6..10 % at N = 4096 and 9216).
        // At N = 1024 the single workgroup per CU this implies leaves the per-workgroup prologue
        // and epilogue uncovered and is slower.
        const bool wide = (g.flags & RIB_FLAG_WIDE) != 0 || (g.N >= 4096 && g.units * (g.N / 512) >= 1024);
        if (g.N % 512 == 0 && wide)
            e = launch_fast<DQK, DVK, 128, 8, XC>(g, q, k, v, fq, fk, out, dout, lse, delta, dq, dk, dv, pq, pk, st);
        else
            e = launch_fast<DQK, DVK, 64, 4, XC>(g, q, k, v, fq, fk, out, dout, lse, delta, dq, dk, dv, pq, pk, st);
        if (e != hipSuccess) return e;
        return launch_reduce_df(g, pq, pk, dfq, dfk, st);
    }
    if constexpr (XC) return hipErrorInvalidValue;   // the general kernels carry the extras in columns only
    if (!g.gate) e = launch_delta(g, RIB_BF16, out, dout, delta, st);     // (gated: done by the caller)
    if (e != hipSuccess) return e;

    const int ntiles = (g.N + kT - 1) / kT;
    const int nblk = (ntiles + kWaves - 1) / kWaves;
    const size_t smem = (size_t)2 * L::STAGE * sizeof(bf16_t) + (size_t)ntiles * kT * sizeof(int);
    if (smem > (size_t)kMaxDynLds) return hipErrorInvalidValue;
    hipError_t pe = prepare_kernel((const void *)mfma_bwd_dq_kernel<DQK, DVK>, nullptr);
    if (pe == hipSuccess) pe = prepare_kernel((const void *)mfma_bwd_dkv_kernel<DQK, DVK>, nullptr);
    if (pe != hipSuccess) return pe;
    const dim3 grid((unsigned)(g.units * nblk)), block(kNT);
    hipLaunchKernelGGL((mfma_bwd_dkv_kernel<DQK, DVK>), grid, block, smem, st, g, nblk, (const bf16_t *)q,
                       (const bf16_t *)k, (const bf16_t *)v, (const bf16_t *)fq, (const bf16_t *)fk,
                       (const bf16_t *)dout, lse, delta, (bf16_t *)dk, (bf16_t *)dv, pk);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((mfma_bwd_dq_kernel<DQK, DVK>), grid, block, smem, st, g, nblk, (const bf16_t *)q,
                       (const bf16_t *)k, (const bf16_t *)v, (const bf16_t *)fq, (const bf16_t *)fk,
                       (const bf16_t *)dout, lse, delta, (bf16_t *)dq, pq);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_reduce_df(g, pq, pk, dfq, dfk, st);
}

}  // namespace

// -LSE and -delta ride either in two spare padding columns of the augmented operands (free
// when d+r+2 and d+2 round up to the same MFMA K multiples as d+r and d) or, on the fast
// path, in the C operand of the score MFMAs, which needs no columns at all: d+r may then
// fill all 64 columns (the paper's r = 34 with d = 30, r = 32 with d = 32) and d all 32.
static bool columns_are_free(const Geo &g)
{
    const int a = g.d + g.r;
    return g.d + 2 <= 32 && (a + 2 <= 48 || (a > 48 && a + 2 <= 64));
}

bool mfma_bwd_supported(const Geo &g, int dtype)
{
    if (!(dtype == RIB_BF16 && !(g.flags & RIB_FLAG_VECTOR_ONLY) && g.d <= 32 && (g.d & 1) == 0 && (g.r & 1) == 0 && g.N >= 64 && g.N <= 9216 &&
          (g.tstride & 1) == 0))
        return false;
    return bwd_fast_ok(g) ? g.d + g.r <= 64 : g.d + g.r + 2 <= 64;
}

hipError_t launch_mfma_bwd(const Geo &g, const void *q, const void *k, const void *v, const void *fq, const void *fk,
                           const void *out, const void *dout, const float *lse, void *dq, void *dk, void *dv,
                           float *dfq, float *dfk, void *ws, hipStream_t st, void *gated_dout, void *dgate)
{
    if (g.gate) {
        float *delta = (float *)((char *)ws + bwd_ws_layout(g).delta_off);
        hipError_t e = launch_delta_gated(g, RIB_BF16, out, dout, g.gate, delta, gated_dout, dgate, st);
        if (e != hipSuccess) return e;
        dout = gated_dout;
    }
    if (bwd_fast_ok(g) && !columns_are_free(g)) {
        // (the 48-column staging code serves RIB rows of up to 32 values)
        if (g.d + g.r <= 48 && g.r <= 32)
            return launch<48, 32, true>(g, q, k, v, fq, fk, out, dout, lse, dq, dk, dv, dfq, dfk, ws, st);
        return launch<64, 32, true>(g, q, k, v, fq, fk, out, dout, lse, dq, dk, dv, dfq, dfk, ws, st);
    }
    const bool small_qk = g.d + g.r + 2 <= 48 && g.r <= 32, small_v = g.d + 2 <= 32;
    if (small_qk && small_v) return launch<48, 32>(g, q, k, v, fq, fk, out, dout, lse, dq, dk, dv, dfq, dfk, ws, st);
    if (small_v) return launch<64, 32>(g, q, k, v, fq, fk, out, dout, lse, dq, dk, dv, dfq, dfk, ws, st);
    return launch<64, 48>(g, q, k, v, fq, fk, out, dout, lse, dq, dk, dv, dfq, dfk, ws, st);
}

}  // namespace rib
