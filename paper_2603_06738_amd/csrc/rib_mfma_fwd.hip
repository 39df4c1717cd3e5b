// RIB window attention, forward, on the gfx950 matrix cores (bf16 MFMA, fp32
// accumulation).  Operator: include/rib_attn.h (paper Sec. 2.2; Sec. 3.1 Eq. 5-6).
//
// Shape of the computation
//   One workgroup = kWaves wavefronts = kWaves*64 consecutive window-local queries
//   of one (window, head) unit.  The unit's keys/values stream through LDS in tiles
//   of 64 tokens (double buffered), gathered from the channel-last grid through a
//   per-workgroup table of token indices that encodes the window partition and
//   the cyclic shift.  K_aug = [k || f_k] rows are assembled in LDS (Eq. 5), the
//   matching Q_aug = [scale_c q || scale_p f_q] rows (pre-multiplied by log2 e)
//   live in registers; neither ever reaches HBM.
//
//   The scores are computed TRANSPOSED, S^T = K_aug Q_aug^T, with the 32x32x16
//   bf16 MFMA: in its accumulator layout a lane owns ONE query column and 16 of
//   the 32 keys, so row maxima and exponentials are lane-local and the packed
//   bf16 probabilities are directly the B operand of the second MFMA,
//   O^T += V^T P^T (keys are visited in the permuted order the accumulator layout
//   implies; V^T is stored in LDS in that order).  The softmax denominator comes
//   out of the same MFMA: V^T carries a row of ones in a padding row of the head
//   dimension (d < 32), so sum_j P_ij accumulates in O^T at no vector-ALU cost.
//
//   Softmax stabiliser.  exp2 of a logit is a normal fp32/bf16 number for any
//   logit in about +-126, so subtracting the row maximum is only needed for
//   extreme logits.  The kernel first runs WITHOUT a stabiliser; afterwards every
//   row checks that its denominator lies in [2^-60, 2^60] (which bounds the largest
//   term and makes flushed terms negligible).  If any row of the workgroup fails,
//   or the caller asks for it, the workgroup redoes its queries with a running
//   maximum that is raised lazily (only when a tile exceeds it by 2^8) and is
//   subtracted for free as the C operand of the score MFMA.  Both paths compute
//   the exact softmax up to rounding.
#include "rib_common.h"

namespace rib {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTK = 64;            // keys per staged tile
constexpr int kVStr = kTK + 8;     // bf16 per V^T row in LDS (144 B: conflict-free 16-byte reads)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLazy = 8.f;       // raise the running max only when exceeded by 2^8

__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    bf16x2 v;
    v[0] = (__bf16)a;
    v[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float lo_bf16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_bf16(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Position of key kappa (0..63) inside a V^T row: within each group of 16 keys the
// order is the one the S^T accumulator layout hands to the PV MFMA.
__device__ __forceinline__ int vt_col(int kappa)
{
    return (kappa & ~15) | (((kappa >> 2) & 1) << 3) | (((kappa >> 3) & 1) << 2) | (kappa & 3);
}

// Row d of O^T (the image of the ones row of V^T = the softmax denominator) for this
// lane's query.  In the accumulator layout it is register 4*(d/8) + d%4 of the half
// (d/4)%2; both halves return it.
__device__ __forceinline__ float ones_row(const f32x16 &O, int d)
{
    const int reg = 4 * (d >> 3) + (d & 3), half = (d >> 2) & 1;
    float mine = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) mine = (i == reg) ? O[i] : mine;
    float other = __shfl_xor(mine, 32);
    return ((int)(threadIdx.x & 63) >> 5) == half ? mine : other;
}

template <int DQK, int WAVES>
struct Stage {
    static constexpr int NT = WAVES * 64;
    static constexpr int KSTR = DQK + 8;               // bf16 per K_aug row in LDS (112 or 144 B)
    static constexpr int CP = kTK * 16 / NT;           // content passes: 16 lanes per token
    static constexpr int FP = (kTK * (DQK / 2) + NT - 1) / NT;  // RIB passes over the flat dword chunk
    uint32_t kc[CP], vc[CP], ff[FP];
};

// Issue the global loads of one 64-token tile (tile index `tile` of tensor x / y,
// RIB table f) into registers.  Tokens past N read nothing and yield zeros.
template <int DQK, int WAVES, bool WITH_V>
__device__ __forceinline__ void tile_load(Stage<DQK, WAVES> &st, const Geo &g, int hd, int tile, const int *tok,
                                          const bf16_t *__restrict__ x, const bf16_t *__restrict__ y,
                                          const bf16_t *__restrict__ f)
{
    using S = Stage<DQK, WAVES>;
    const int tid = threadIdx.x;
    const int pair = tid & 15;
#pragma unroll
    for (int p = 0; p < S::CP; ++p) {
        int nl = p * (S::NT / 16) + (tid >> 4);
        int t = tok[tile * kTK + nl];
        uint32_t a = 0, b = 0;
        if (t >= 0 && 2 * pair < g.d) {
            int64_t off = (int64_t)t * g.tstride + hd * g.d + 2 * pair;
            a = *(const uint32_t *)(x + off);
            if (WITH_V) b = *(const uint32_t *)(y + off);
        }
        st.kc[p] = a;
        st.vc[p] = b;
    }
    const int n0 = tile * kTK;
    const int live = (g.N - n0 < kTK ? g.N - n0 : kTK) * (g.r >> 1);
    const uint32_t *fsrc = (const uint32_t *)(f + ((int64_t)hd * g.N + n0) * g.r);
#pragma unroll
    for (int p = 0; p < S::FP; ++p) {
        int e = p * S::NT + tid;
        st.ff[p] = (e < live) ? fsrc[e] : 0u;
    }
}

// Write a loaded tile into LDS: K_aug rows [64][KSTR] (content scaled by sc, RIB
// part by sp when SCALE) and, when WITH_V, V^T [32][kVStr] in permuted key order.
template <int DQK, int WAVES, bool WITH_V, bool SCALE>
__device__ __forceinline__ void tile_store(const Stage<DQK, WAVES> &st, const Geo &g, bf16_t *Ka, bf16_t *Vt, float sc,
                                           float sp, const int *foff)
{
    using S = Stage<DQK, WAVES>;
    const int tid = threadIdx.x;
    const int pair = tid & 15;
#pragma unroll
    for (int p = 0; p < S::CP; ++p) {
        int nl = p * (S::NT / 16) + (tid >> 4);
        if (2 * pair < g.d) {
            uint32_t a = st.kc[p];
            if (SCALE) a = pack_bf16(lo_bf16(a) * sc, hi_bf16(a) * sc);
            *(uint32_t *)(Ka + nl * S::KSTR + 2 * pair) = a;
            if (WITH_V) {
                int col = vt_col(nl);
                Vt[(2 * pair) * kVStr + col] = (bf16_t)(st.vc[p] & 0xffffu);
                Vt[(2 * pair + 1) * kVStr + col] = (bf16_t)(st.vc[p] >> 16);
            }
        }
    }
    const int fdw = kTK * (g.r >> 1);
#pragma unroll
    for (int p = 0; p < S::FP; ++p) {
        int e = p * S::NT + tid;
        if (e < fdw) {
            uint32_t a = st.ff[p];
            if (SCALE) a = pack_bf16(lo_bf16(a) * sp, hi_bf16(a) * sp);
            *(uint32_t *)(Ka + foff[p]) = a;
        }
    }
}

// One pass of a wave's 64 queries over all keys of the unit.
template <int DQK, int WAVES, bool ONES, bool TRACK_MAX>
__device__ __forceinline__ void attend(const Geo &g, int hd, const int *tok, bf16_t (*Ka)[kTK * (DQK + 8)],
                                       bf16_t (*Vt)[32 * kVStr], const int *foff, const bf16x8 (&Q)[2][DQK / 16],
                                       const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                       const bf16_t *__restrict__ fk, f32x16 (&O)[2], float (&mrun)[2], float (&lsum)[2])
{
    constexpr int KS = DQK / 16;
    constexpr int KSTR = DQK + 8;
    const int lane = threadIdx.x & 63;
    const int col = lane & 31, hf = lane >> 5;
    const int ntiles = (g.N + kTK - 1) / kTK;
    const bool ragged = (g.N % kTK) != 0;

    f32x16 negM[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { O[qb][i] = 0.f; negM[qb][i] = 0.f; }
        mrun[qb] = 0.f;
        lsum[qb] = 0.f;
    }

    Stage<DQK, WAVES> st;
    tile_load<DQK, WAVES, true>(st, g, hd, 0, tok, k, v, fk);
    tile_store<DQK, WAVES, true, false>(st, g, Ka[0], Vt[0], 1.f, 1.f, foff);
    __syncthreads();

    for (int tile = 0; tile < ntiles; ++tile) {
        const int cur = tile & 1;
        if (tile + 1 < ntiles) tile_load<DQK, WAVES, true>(st, g, hd, tile + 1, tok, k, v, fk);
        const bool last_ragged = ragged && (tile == ntiles - 1);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            bf16x8 Ak[KS], Av[2];
#pragma unroll
            for (int t = 0; t < KS; ++t)
                Ak[t] = *(const bf16x8 *)(Ka[cur] + (kb * 32 + col) * KSTR + 16 * t + 8 * hf);
#pragma unroll
            for (int t = 0; t < 2; ++t)
                Av[t] = *(const bf16x8 *)(Vt[cur] + col * kVStr + kb * 32 + 16 * t + 8 * hf);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                f32x16 S;
                if (TRACK_MAX) S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ak[0], Q[qb][0], negM[qb], 0, 0, 0);
                else {
                    f32x16 z = {0};
                    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ak[0], Q[qb][0], z, 0, 0, 0);
                }
#pragma unroll
                for (int t = 1; t < KS; ++t) S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ak[t], Q[qb][t], S, 0, 0, 0);
                if (last_ragged) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        int key = tile * kTK + kb * 32 + 8 * (i >> 2) + 4 * hf + (i & 3);
                        if (key >= g.N) S[i] = -INFINITY;
                    }
                }
                if (TRACK_MAX) {
                    // S holds logit - mrun.  Raise mrun when some logit exceeds it by 2^kLazy
                    // (always on the very first block, where mrun is still a placeholder).
                    float tm = fmaxf(fmaxf(S[0], S[1]), S[2]);
#pragma unroll
                    for (int i = 3; i < 15; i += 2) tm = fmaxf(fmaxf(tm, S[i]), S[i + 1]);
                    tm = fmaxf(tm, S[15]);
                    tm = fmaxf(tm, __shfl_xor(tm, 32));
                    const bool first = (tile == 0 && kb == 0);
                    bool need = first || tm > kLazy;
                    if (__any(need)) {
                        float delta = need ? tm : 0.f;              // new mrun = mrun + delta
                        if (delta == -INFINITY) delta = 0.f;
                        float alpha = __builtin_amdgcn_exp2f(fminf(-delta, 126.f));
                        mrun[qb] += delta;
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            S[i] -= delta;
                            O[qb][i] *= alpha;
                            negM[qb][i] = -mrun[qb];
                        }
                        lsum[qb] *= alpha;
                    }
                }
                float p[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) p[i] = __builtin_amdgcn_exp2f(S[i]);
                if (!ONES) {
                    float a = 0.f;
#pragma unroll
                    for (int i = 0; i < 16; ++i) a += p[i];
                    lsum[qb] += a;
                }
                bf16x8 P0, P1;
#pragma unroll
                for (int i = 0; i < 8; ++i) { P0[i] = (__bf16)p[i]; P1[i] = (__bf16)p[8 + i]; }
                O[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Av[0], P0, O[qb], 0, 0, 0);
                O[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Av[1], P1, O[qb], 0, 0, 0);
            }
        }
        if (tile + 1 < ntiles) tile_store<DQK, WAVES, true, false>(st, g, Ka[cur ^ 1], Vt[cur ^ 1], 1.f, 1.f, foff);
        __syncthreads();
    }
}

template <int DQK, int WAVES, bool ONES>
__global__ __launch_bounds__(WAVES * 64, WAVES == 4 ? 2 : 1) void mfma_fwd_kernel(
    Geo g, int nqblk, int force_max, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
    const bf16_t *__restrict__ v, const bf16_t *__restrict__ fq, const bf16_t *__restrict__ fk,
    bf16_t *__restrict__ out, float *__restrict__ lse)
{
    constexpr int NT = WAVES * 64;
    constexpr int KS = DQK / 16;
    constexpr int KSTR = DQK + 8;
    using St = Stage<DQK, WAVES>;
    __shared__ __attribute__((aligned(16))) bf16_t Ka[2][kTK * KSTR];
    __shared__ __attribute__((aligned(16))) bf16_t Vt[2][32 * kVStr];
    extern __shared__ int tok[];   // [ntiles*64] grid token of each window-local token, -1 past N

    // Workgroups are dealt round-robin to the 8 XCDs; renumber them so that each XCD
    // works on a contiguous range of (unit, query block) and its L2 sees all users
    // of a window's K/V lines.
    const int G = gridDim.x, per = G >> 3, rem = G & 7, xcd = blockIdx.x & 7;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    const int64_t u = logical / nqblk;
    const int blk = logical - (int)(u * nqblk);
    const int w = (int)(u / g.heads), hd = (int)(u - (int64_t)w * g.heads);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, hf = lane >> 5;
    const int ntiles = (g.N + kTK - 1) / kTK;

    for (int n = tid; n < ntiles * kTK; n += NT) tok[n] = n < g.N ? (int)grid_token(g, w, n) : -1;
    // constant parts of the LDS tiles: zero padding columns of K_aug, the ones row and
    // zero rows of V^T (the staging code never writes them)
    for (int e = tid; e < 2 * kTK * KSTR; e += NT) {
        int c = e % KSTR;
        if (c >= g.d + g.r) Ka[0][e] = 0;
    }
    for (int e = tid; e < 2 * 32 * kVStr; e += NT) {
        int row = (e % (32 * kVStr)) / kVStr;
        if (row >= g.d) Vt[0][e] = (ONES && row == g.d) ? (bf16_t)0x3f80 : (bf16_t)0;
    }
    int foff[St::FP];
#pragma unroll
    for (int p = 0; p < St::FP; ++p) {
        int e = p * NT + tid, hr = g.r >> 1;
        int tk = hr > 0 ? e / hr : 0;
        foff[p] = tk * KSTR + g.d + 2 * (e - tk * hr);
    }
    __syncthreads();

    // Q_aug of this wave's 64 queries -> B operands, staged through LDS one wave at a time
    bf16x8 Q[2][KS];
    {
        const float sc = g.scale_c * kLog2e, sp = g.scale_p * kLog2e;
        St st;
        for (int wv = 0; wv < WAVES; ++wv) {
            int qtile = (blk * NT + wv * 64) / kTK;     // query blocks are tile aligned (NT % 64 == 0)
            if (qtile < ntiles) {
                tile_load<DQK, WAVES, false>(st, g, hd, qtile, tok, q, q, fq);
                tile_store<DQK, WAVES, false, true>(st, g, Ka[0], Vt[0], sc, sp, foff);
            }
            __syncthreads();
            if (wv == wave && qtile < ntiles) {
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int t = 0; t < KS; ++t)
                        Q[qb][t] = *(const bf16x8 *)(Ka[0] + (qb * 32 + col) * KSTR + 16 * t + 8 * hf);
            }
            __syncthreads();
        }
    }
    const int q0 = blk * NT + wave * 64;               // first query of this wave
    if (q0 >= g.N) {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int t = 0; t < KS; ++t)
#pragma unroll
                for (int i = 0; i < 8; ++i) Q[qb][t][i] = (__bf16)0.f;
    }

    f32x16 O[2];
    float mrun[2], lsum[2];
    bool redo = force_max != 0;
    if (!redo) {
        attend<DQK, WAVES, ONES, false>(g, hd, tok, Ka, Vt, foff, Q, k, v, fk, O, mrun, lsum);
        bool bad = false;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float l = ONES ? ones_row(O[qb], g.d) : lsum[qb] + __shfl_xor(lsum[qb], 32);
            bool ok = (l >= 0x1p-60f) && (l <= 0x1p60f);
            if (!ok && q0 + qb * 32 + col < g.N) bad = true;
        }
        redo = __syncthreads_or(bad);
    }
    if (redo) attend<DQK, WAVES, ONES, true>(g, hd, tok, Ka, Vt, foff, Q, k, v, fk, O, mrun, lsum);

    // normalise and scatter through the inverse window map
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float l;
        if (ONES) {
            l = ones_row(O[qb], g.d);
        } else {
            l = lsum[qb] + __shfl_xor(lsum[qb], 32);
        }
        const int n = q0 + qb * 32 + col;
        if (n >= g.N) continue;
        const float inv = 1.f / l;
        bf16_t *dst = out + (int64_t)tok[n] * g.C + hd * g.d;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            int dv = 8 * (i >> 2) + 4 * hf + (i & 3);
            if (dv < g.d) *(uint32_t *)(dst + dv) = pack_bf16(O[qb][i] * inv, O[qb][i + 1] * inv);
        }
        if (lse != nullptr && hf == 0) lse[u * g.N + n] = (mrun[qb] + __builtin_amdgcn_logf(l)) * kLn2;
    }
}

template <int DQK, bool ONES>
hipError_t launch(const Geo &g, int force_max, const void *q, const void *k, const void *v, const void *fq,
                  const void *fk, void *out, float *lse, hipStream_t st)
{
    constexpr int WAVES = 4;
    const int nqblk = (g.N + WAVES * 64 - 1) / (WAVES * 64);
    const int ntiles = (g.N + kTK - 1) / kTK;
    const size_t dyn = (size_t)ntiles * kTK * sizeof(int);
    hipLaunchKernelGGL((mfma_fwd_kernel<DQK, WAVES, ONES>), dim3((unsigned)(g.units * nqblk)), dim3(WAVES * 64), dyn,
                       st, g, nqblk, force_max, (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v,
                       (const bf16_t *)fq, (const bf16_t *)fk, (bf16_t *)out, lse);
    return hipGetLastError();
}

}  // namespace

bool mfma_fwd_supported(const Geo &g, int dtype)
{
    return dtype == RIB_BF16 && g.d <= 32 && (g.d & 1) == 0 && (g.r & 1) == 0 && g.d + g.r <= 64 && g.N >= 64 &&
           g.N <= 9216 && (g.tstride & 1) == 0;
}

hipError_t launch_mfma_fwd(const Geo &g, int force_max, const void *q, const void *k, const void *v, const void *fq,
                           const void *fk, void *out, float *lse, hipStream_t st)
{
    const bool ones = g.d < 32;
    if (g.d + g.r <= 48)
        return ones ? launch<48, true>(g, force_max, q, k, v, fq, fk, out, lse, st)
                    : launch<48, false>(g, force_max, q, k, v, fq, fk, out, lse, st);
    return ones ? launch<64, true>(g, force_max, q, k, v, fq, fk, out, lse, st)
                : launch<64, false>(g, force_max, q, k, v, fq, fk, out, lse, st);
}

}  // namespace rib
