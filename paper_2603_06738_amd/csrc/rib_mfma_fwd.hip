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
#include <mutex>

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
// Two fp32 -> one dword of two bf16 by dropping the low 16 bits (round toward zero).
__device__ __forceinline__ uint32_t trunc_pack(float lo, float hi)
{
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}
__device__ __forceinline__ bf16x8 as_bf16x8(const uint4 &w) { return __builtin_bit_cast(bf16x8, w); }
// Mean relative loss of truncating to bf16 (spacing 2^-7, mantissa log-uniform in [1,2)):
// 2^-8 / (2 ln 2) * ... = 2^-8 * 0.7213; as a log2 it is added back to the softmax denominator's log.
constexpr float kTruncLog2 = 0.0040593f;
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
template <int DQK, int WAVES, bool WITH_V, class TK>
__device__ __forceinline__ void tile_load(Stage<DQK, WAVES> &st, const Geo &g, int hd, int tile, const TK &tok,
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
template <int DQK, int WAVES, bool ONES, bool TRACK_MAX, class TK>
__device__ __forceinline__ void attend(const Geo &g, int hd, const TK &tok, bf16_t (*Ka)[kTK * (DQK + 8)],
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


// ---------------------------------------------------------------------------------------
// Fast path: full tiles of 128 keys, no masking, no running maximum, and a hand-ordered
// software pipeline.  For the 32x32 block s of a tile the wave issues, interleaved,
//   the 3 score MFMAs of block s+1, the 16 exp2 + 8 bf16 packs of block s, and the
//   2 PV MFMAs of block s-1,
// so the matrix pipe and the vector ALU work on independent data all the time; the
// staging of the next tile (global loads early, LDS writes late) rides in the gaps.
// Scheduling fences keep the compiler from regrouping the instruction stream.
// The fast path runs with 4 or 8 waves per workgroup; a K/V tile holds 32 keys per wave (128 or
// 256), so that one pass of the staging code (8 lanes per token, 4 tokens per thread) fills it.
template <int WAVES>
struct FastTile {
    static constexpr int FT = 32 * WAVES;       // keys per tile
    static constexpr int FVS = FT + 8;          // bf16 per V^T row (272 / 528 B: conflict-free 16-byte reads)
};
// scheduling-group masks of __builtin_amdgcn_sched_group_barrier
#define RIB_SG_VALU 0x002
#define RIB_SG_MFMA 0x008
#define RIB_SG_VMEM_RD 0x020
#define RIB_SG_DS_RD 0x100
#define RIB_SG_DS_WR 0x200
#define RIB_SG_TRANS 0x400
#define RIB_SG(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)

// Emits, for m = M0 .. M1-1: one MFMA, then 3 or 4 transcendentals (16 per 5 MFMAs),
// then 2 vector-ALU instructions.
template <int M0, int M1>
__device__ __forceinline__ void sched_pipeline()
{
    if constexpr (M0 < M1) {
        RIB_SG(RIB_SG_MFMA, 1);
        RIB_SG(RIB_SG_TRANS, (M0 % 5) == 4 ? 4 : 3);
        RIB_SG(RIB_SG_VALU, 2);
        sched_pipeline<M0 + 1, M1>();
    }
}

// Two dwords at a 4-byte aligned address (global memory only needs dword alignment for
// multi-dword accesses; LDS gets them as a two-dword write).
struct __attribute__((packed, aligned(4))) dword2 {
    uint32_t x, y;
};

// Staging registers of one 128-token tile: 8 lanes share a token and each thread serves 4
// consecutive tokens, with 8 bytes per tensor per token.
template <int DQK>
struct FastRegs {
    dword2 kx[4], vx[4], fa[4];
    dword2 fb[DQK == 64 ? 4 : 1];       // second RIB slot: rows longer than 32 values
};

template <int DQK>
struct FastConst {                  // per-thread staging constants
    uint32_t lane_c;                // byte offset of this lane's two content dwords inside a token
    uint32_t tsb;                   // token stride in bytes
    int tok_idx;                    // first of this lane's 4 tokens inside a tile
    uint32_t f_off0, f_off1;        // byte offsets of this lane's RIB dword pairs inside a RIB row
    int k_dst, f_dst0, f_dst1, v_dst;   // bf16 element offsets inside a stage
};

template <int DQK, int WAVES>
__device__ __forceinline__ FastConst<DQK> fast_const(const Geo &g, int hd)
{
    constexpr int KSTR = DQK + 8, kFVS = FastTile<WAVES>::FVS;
    FastConst<DQK> c;
    const int tid = threadIdx.x, grp = tid >> 3, j = tid & 7;
    const int hp = g.d >> 1, rh = g.r >> 1;             // dwords per content row / RIB row (both >= 2)
    // lane j serves dwords 2j, 2j+1; lanes past the end slide back onto the last pair (their
    // loads and stores then duplicate a neighbour's, which is harmless)
    const int dj = 2 * j + 1 < hp ? 2 * j : hp - 2;
    const int f0 = 2 * j + 1 < rh ? 2 * j : rh - 2;
    const int f1 = 16 + 2 * j + 1 < rh ? 16 + 2 * j : rh - 2;
    c.lane_c = (uint32_t)(hd * g.d + 2 * dj) * 2u;
    c.tsb = (uint32_t)g.tstride * 2u;
    c.tok_idx = grp * 4;
    c.f_off0 = (uint32_t)f0 * 4u;
    c.f_off1 = (uint32_t)f1 * 4u;
    c.k_dst = grp * 4 * KSTR + 2 * dj;
    c.f_dst0 = grp * 4 * KSTR + g.d + 2 * f0;
    c.f_dst1 = grp * 4 * KSTR + g.d + 2 * f1;
    // V^T rows 2dj .. 2dj+3; the 4 tokens of this lane sit at permuted columns pc .. pc+3
    const int nl = grp * 4;
    const int pc = (nl & ~15) | (((nl >> 2) & 1) << 3) | (((nl >> 3) & 1) << 2);
    c.v_dst = (2 * dj) * kFVS + pc;
    return c;
}

// global loads of this lane's four tokens of the tile that starts at window-local token n0
template <int DQK>
__device__ __forceinline__ void fast_load(FastRegs<DQK> &rg, const FastConst<DQK> &c, const Geo &g, const TokMap &tok, int n0,
                                          const char *kb, const char *vb, const char *fb)
{
    int t[4];
    tok.quad(n0 + c.tok_idx, t);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t off = __umul24((uint32_t)t[p], c.tsb) + c.lane_c;
        rg.kx[p] = *(const dword2 *)(kb + off);
        rg.vx[p] = *(const dword2 *)(vb + off);
        const uint32_t row = (uint32_t)(c.tok_idx + p) * (uint32_t)(g.r * 2);
        rg.fa[p] = *(const dword2 *)(fb + row + c.f_off0);
        if (DQK == 64) rg.fb[p] = *(const dword2 *)(fb + row + c.f_off1);
    }
}

// LDS writes of token p: its pieces of the K_aug row; after the 4th token the four V^T
// rows of this lane (4 keys per 8-byte write)
template <int DQK, int WAVES>
__device__ __forceinline__ void fast_store(const FastRegs<DQK> &rg, const FastConst<DQK> &c, int p, bf16_t *Kf, bf16_t *Vf)
{
    constexpr int KSTR = DQK + 8, kFVS = FastTile<WAVES>::FVS;
    *(dword2 *)(Kf + c.k_dst + p * KSTR) = rg.kx[p];
    *(dword2 *)(Kf + c.f_dst0 + p * KSTR) = rg.fa[p];
    if (DQK == 64) *(dword2 *)(Kf + c.f_dst1 + p * KSTR) = rg.fb[p];
    if (p == 3) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t a = h ? rg.vx[0].y : rg.vx[0].x, b = h ? rg.vx[1].y : rg.vx[1].x;
            const uint32_t cc = h ? rg.vx[2].y : rg.vx[2].x, d = h ? rg.vx[3].y : rg.vx[3].x;
            uint2 even, odd;
            even.x = __builtin_amdgcn_perm(b, a, 0x05040100u);
            even.y = __builtin_amdgcn_perm(d, cc, 0x05040100u);
            odd.x = __builtin_amdgcn_perm(b, a, 0x07060302u);
            odd.y = __builtin_amdgcn_perm(d, cc, 0x07060302u);
            *(uint2 *)(Vf + c.v_dst + (2 * h) * kFVS) = even;
            *(uint2 *)(Vf + c.v_dst + (2 * h + 1) * kFVS) = odd;
        }
    }
}

// Byte bases and per-thread constants the fast staging needs.
template <int DQK>
struct FastCtx {
    FastConst<DQK> c;
    const char *kbase, *vbase, *fbase;
    uint32_t ftile;                 // bytes of RIB rows per tile
};
template <int DQK, int WAVES>
__device__ __forceinline__ FastCtx<DQK> fast_ctx(const Geo &g, int hd, const bf16_t *k, const bf16_t *v, const bf16_t *fk)
{
    constexpr int kFT = FastTile<WAVES>::FT;
    FastCtx<DQK> x;
    x.c = fast_const<DQK, WAVES>(g, hd);
    x.kbase = (const char *)k;
    x.vbase = (const char *)v;
    x.fbase = (const char *)(fk + (int64_t)hd * g.N * g.r);
    x.ftile = (uint32_t)kFT * (uint32_t)(g.r * 2);
    return x;
}

// `rg` holds tile 0 (its global loads were issued by the caller, early).
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#define kOnes2 __builtin_bit_cast(bf16x2, 0x3f803f80u)

template <int DQK, bool ONES, int WAVES>
__device__ __forceinline__ void attend_fast(const Geo &g, const FastCtx<DQK> &fx, FastRegs<DQK> &rg, const TokMap &tok,
                                            bf16_t *Kf, bf16_t *Vf, const bf16x8 (&Q)[2][DQK / 16], f32x16 (&O)[2],
                                            float (&lsum)[2])
{
    constexpr int KS = DQK / 16, KSTR = DQK + 8;
    constexpr int kFT = FastTile<WAVES>::FT, kFVS = FastTile<WAVES>::FVS;
    constexpr int NKB = kFT / 32, NSTEP = 2 * NKB;        // key blocks per tile; (key block, query block) steps
    constexpr int KSZ = kFT * KSTR, VSZ = 32 * kFVS;     // bf16 per stage
    const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
    const int ntiles = g.N / kFT;
    const FastConst<DQK> &c = fx.c;
    const char *kbase = fx.kbase, *vbase = fx.vbase, *fbase = fx.fbase;
    const uint32_t ftile = fx.ftile;

#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) O[qb][i] = 0.f;
        lsum[qb] = 0.f;
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) fast_store<DQK, WAVES>(rg, c, p, Kf, Vf);
    {   // tile 1 goes in flight now and is written to LDS at the end of tile 0's block
        const int t1 = ntiles > 1 ? 1 : 0;
        fast_load<DQK>(rg, c, g, tok, t1 * kFT, kbase, vbase, fbase + (uint32_t)t1 * ftile);
    }
    __syncthreads();

    const f32x16 zero = {0};
    for (int tile = 0; tile < ntiles; ++tile) {
        const int cur = tile & 1;
        const bf16_t *Kc = Kf + cur * KSZ, *Vc = Vf + cur * VSZ;
        bf16_t *Kn = Kf + (cur ^ 1) * KSZ, *Vn = Vf + (cur ^ 1) * VSZ;
        // `rg` holds tile+1 (requested one block ago); tile+2 is requested at the end of this
        // block.  Past the end both clamp to the last tile (staged again, never used).
        const int nt = tile + 2 < ntiles ? tile + 2 : ntiles - 1;
        const char *fn = fbase + (uint32_t)nt * ftile;

        bf16x8 Ak[NKB][KS], Av[NKB][2];
        f32x16 S[2];
        uint4 P[2][2];          // packed bf16 probabilities: B operands of the PV MFMAs
#pragma unroll
        for (int t = 0; t < KS; ++t) Ak[0][t] = *(const bf16x8 *)(Kc + col * KSTR + 16 * t + 8 * hf);
#pragma unroll
        for (int t = 0; t < 2; ++t) Av[0][t] = *(const bf16x8 *)(Vc + col * kFVS + 16 * t + 8 * hf);
        S[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ak[0][0], Q[0][0], zero, 0, 0, 0);
#pragma unroll
        for (int t = 1; t < KS; ++t) S[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ak[0][t], Q[0][t], S[0], 0, 0, 0);

#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            const int kb = s >> 1, qb = s & 1, cs = s & 1, ns = cs ^ 1;
            const int s1 = s + 1, kb1 = s1 >> 1, qb1 = s1 & 1;
            const int kbp = (s - 1) >> 1, qbp = (s - 1) & 1;
            float pe[16];
            // group 0..2: one score MFMA of the next block + 4 exp2 and 2 packs of this block
#pragma unroll
            for (int grp = 0; grp < 4; ++grp) {
                if (grp < 3) {
                    if (s < NSTEP - 1 && grp < 2) {
                        S[ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ak[kb1][grp], Q[qb1][grp],
                                                                         grp == 0 ? zero : S[ns], 0, 0, 0);
                    }
                    if (s < NSTEP - 1 && grp == 2) {
#pragma unroll
                        for (int t = 2; t < KS; ++t)
                            S[ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ak[kb1][t], Q[qb1][t], S[ns], 0, 0, 0);
                    }
                } else if (s > 0) {
                    O[qbp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Av[kbp][0], as_bf16x8(P[ns][0]), O[qbp], 0, 0, 0);
                }
#pragma unroll
                for (int i = 4 * grp; i < 4 * grp + 4; ++i) pe[i] = __builtin_amdgcn_exp2f(S[cs][i]);
                // fp32 -> bf16 by truncation: one byte-permute per pair instead of the (slow)
                // rounding convert.  Numerator and denominator use the same truncated P.
                const uint32_t w0 = trunc_pack(pe[4 * grp], pe[4 * grp + 1]);
                const uint32_t w1 = trunc_pack(pe[4 * grp + 2], pe[4 * grp + 3]);
                if (!ONES) {    // no spare V^T row for the ones: sum the packed pairs with the bf16 dot product
                    lsum[qb] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w0), kOnes2, lsum[qb], false);
                    lsum[qb] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w1), kOnes2, lsum[qb], false);
                }
                if ((grp & 1) == 0) {
                    P[cs][grp >> 1].x = w0;
                    P[cs][grp >> 1].y = w1;
                } else {
                    P[cs][grp >> 1].z = w0;
                    P[cs][grp >> 1].w = w1;
                }
            }
            // group 4: second PV MFMA of the previous block + this step's share of the staging
            if (s > 0) O[qbp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Av[kbp][1], as_bf16x8(P[ns][1]), O[qbp], 0, 0, 0);
            if (qb == 0 && kb + 1 < NKB) {
#pragma unroll
                for (int t = 0; t < KS; ++t)
                    Ak[kb + 1][t] = *(const bf16x8 *)(Kc + ((kb + 1) * 32 + col) * KSTR + 16 * t + 8 * hf);
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    Av[kb + 1][t] = *(const bf16x8 *)(Vc + col * kFVS + (kb + 1) * 32 + 16 * t + 8 * hf);
            }
        }
        // drain: PV of the last block
        O[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Av[NKB - 1][0], as_bf16x8(P[1][0]), O[1], 0, 0, 0);
        O[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Av[NKB - 1][1], as_bf16x8(P[1][1]), O[1], 0, 0, 0);
        // staging of the next tiles: tile+1 (requested a whole block ago) goes to LDS, then
        // tile+2 is requested into the same registers
#pragma unroll
        for (int p = 0; p < 4; ++p) fast_store<DQK, WAVES>(rg, c, p, Kn, Vn);
        fast_load<DQK>(rg, c, g, tok, nt * kFT, kbase, vbase, fn);

        // The order the scheduler is asked to build out of the block above: every MFMA
        // followed by its share of the exp2 (transcendental) and pack (VALU) work.
        sched_pipeline<0, NSTEP * (DQK / 16 + 2)>();
        __syncthreads();
    }
}

// Constant parts of the generic (64-key) LDS tiles: zero padding columns of K_aug, the
// ones row and the zero rows of V^T.  The staging code never writes them.
template <int DQK, int NT, bool ONES>
__device__ __forceinline__ void init_generic_tiles(const Geo &g, bf16_t *Ka, bf16_t *Vt)
{
    constexpr int KSTR = DQK + 8;
    for (int e = threadIdx.x; e < 2 * kTK * KSTR; e += NT)
        if (e % KSTR >= g.d + g.r) Ka[e] = 0;
    for (int e = threadIdx.x; e < 2 * 32 * kVStr; e += NT) {
        int row = (e % (32 * kVStr)) / kVStr;
        if (row >= g.d) Vt[e] = (ONES && row == g.d) ? (bf16_t)0x3f80 : (bf16_t)0;
    }
}
template <int DQK, int NT, bool ONES>
__device__ __forceinline__ void init_fast_tiles(const Geo &g, bf16_t *Kf, bf16_t *Vf)
{
    constexpr int KSTR = DQK + 8, kFT = FastTile<NT / 64>::FT, kFVS = FastTile<NT / 64>::FVS;
    const int pad0 = g.d + g.r;                                  // even; columns pad0..DQK-1 are zero
    for (int row = threadIdx.x; row < 2 * kFT; row += NT)
        for (int c = pad0; c < DQK; c += 2) *(uint32_t *)(Kf + row * KSTR + c) = 0u;
    const int vrows = 32 - g.d;                                  // rows d..31 of both stages
    for (int e = threadIdx.x; e < 2 * vrows * (kFVS / 2); e += NT) {
        const int per = vrows * (kFVS / 2);
        const int st = e / per, rem = e - st * per;
        const int row = g.d + rem / (kFVS / 2), cw = rem - (rem / (kFVS / 2)) * (kFVS / 2);
        *(uint32_t *)(Vf + (st * 32 + row) * kFVS + 2 * cw) = (ONES && row == g.d) ? 0x3f803f80u : 0u;
    }
}

template <int DQK, bool FAST, int WAVES = 4>
struct FwdSmem {
    static constexpr int KSTR = DQK + 8;
    static constexpr int GEN_K = 2 * kTK * KSTR, GEN_V = 2 * 32 * kVStr;       // bf16 elements
    static constexpr int FAST_K = 2 * FastTile<WAVES>::FT * KSTR, FAST_V = 2 * 32 * FastTile<WAVES>::FVS;
    static constexpr int TILE_ELEMS = FAST ? (FAST_K + FAST_V) : (GEN_K + GEN_V);
    static constexpr size_t TILE_BYTES = (size_t)TILE_ELEMS * sizeof(bf16_t);
};

template <int DQK, int WAVES, bool ONES, bool FAST>
__global__ __launch_bounds__(WAVES * 64, 2) void mfma_fwd_kernel(
    Geo g, int nqblk, int force_max, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
    const bf16_t *__restrict__ v, const bf16_t *__restrict__ fq, const bf16_t *__restrict__ fk,
    bf16_t *__restrict__ out, float *__restrict__ lse)
{
    constexpr int NT = WAVES * 64;
    constexpr int KS = DQK / 16;
    constexpr int KSTR = DQK + 8;
    using St = Stage<DQK, WAVES>;
    using Sm = FwdSmem<DQK, FAST>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *tiles = (bf16_t *)smem;
    bf16_t(*Ka)[kTK * KSTR] = (bf16_t(*)[kTK * KSTR]) tiles;                   // generic layout
    bf16_t(*Vt)[32 * kVStr] = (bf16_t(*)[32 * kVStr])(tiles + Sm::GEN_K);
    int *tok = (int *)(smem + Sm::TILE_BYTES);   // [ntiles*64] grid token of each window-local token, -1 past N

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

    fill_tok_table<NT>(g, w, tok, ntiles * kTK);
    init_generic_tiles<DQK, NT, ONES>(g, Ka[0], Vt[0]);
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
    float mrun[2] = {0.f, 0.f}, lsum[2];
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
        const int64_t obase = (int64_t)tok[n] * g.C + hd * g.d;
        bf16_t *dst = out + obase;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            int dv = 8 * (i >> 2) + 4 * hf + (i & 3);
            if (dv >= g.d) continue;
            const float o0 = O[qb][i] * inv, o1 = O[qb][i + 1] * inv;
            if (g.gate == nullptr) {
                *(uint32_t *)(dst + dv) = pack_bf16(o0, o1);
            } else {    // CLA gate (Eq. 9) on the way out, the raw O beside it if asked for
                const uint32_t gw = *(const uint32_t *)((const bf16_t *)g.gate + obase + dv);
                *(uint32_t *)(dst + dv) = pack_bf16(o0 * lo_bf16(gw), o1 * hi_bf16(gw));
                if (g.out_raw) *(uint32_t *)((bf16_t *)g.out_raw + obase + dv) = pack_bf16(o0, o1);
            }
        }
        if (lse != nullptr && hf == 0) lse[u * g.N + n] = (mrun[qb] + __builtin_amdgcn_logf(l)) * kLn2;
    }
}

// Forward kernel for the common case (whole 128-key tiles, 32-bit byte offsets, r > 0):
// a prologue with ONE exposed global-memory latency (the first K/V tile and all Q rows
// are requested together; each wave stages its own 64 Q_aug rows), then attend_fast.
// Rows whose softmax denominator leaves the safe range send the workgroup through the
// max-tracking path of the general kernel.
template <int DQK, bool ONES, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 2) void mfma_fwd_fast_kernel(
    Geo g, int nqblk, int force_max, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
    const bf16_t *__restrict__ v, const bf16_t *__restrict__ fq, const bf16_t *__restrict__ fk,
    bf16_t *__restrict__ out, float *__restrict__ lse)
{
    constexpr int NT = WAVES * 64;
    constexpr int kFT = FastTile<WAVES>::FT, kFVS = FastTile<WAVES>::FVS;
    constexpr int KS = DQK / 16;
    constexpr int KSTR = DQK + 8;
    using St = Stage<DQK, WAVES>;
    using Sm = FwdSmem<DQK, true, WAVES>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    bf16_t *tiles = (bf16_t *)smem;
    bf16_t *Kf = tiles, *Vf = tiles + Sm::FAST_K;
    // (window-local token -> grid token, as two tables of M entries)

    const int G = gridDim.x, per = G >> 3, rem = G & 7, xcd = blockIdx.x & 7;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    const int64_t u = logical / nqblk;
    const int blk = logical - (int)(u * nqblk);
    const int w = (int)(u / g.heads), hd = (int)(u - (int64_t)w * g.heads);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, hf = lane >> 5;

    const TokMap tok = fill_tok_map<NT>(g, w, (int *)(smem + Sm::TILE_BYTES));
    {   // zero the Q staging area (rows of all four waves): its padding columns must read 0
        uint4 z = {0u, 0u, 0u, 0u};
        for (int e = tid; e < NT * KSTR / 8; e += NT) ((uint4 *)tiles)[e] = z;
    }
    __syncthreads();

    const FastCtx<DQK> fx = fast_ctx<DQK, WAVES>(g, hd, k, v, fk);
    FastRegs<DQK> rg;
    fast_load<DQK>(rg, fx.c, g, tok, 0, fx.kbase, fx.vbase, fx.fbase);

    // Q_aug rows of this wave: 16 lanes per token, 4 tokens per pass
    const int q0 = blk * NT + wave * 64;
    bf16x8 Q[2][KS];
    {
        const float sc = g.scale_c * kLog2e, sp = g.scale_p * kLog2e;
        const int sub = lane >> 4, j = lane & 15, hp = g.d >> 1, rh = g.r >> 1;
        const int pair = j < hp ? j : hp - 1;
        const int f0 = j < rh ? j : rh - 1, f1 = 16 + j < rh ? 16 + j : rh - 1;
        const char *qbase = (const char *)q;
        const char *fqb = (const char *)(fq + ((int64_t)hd * g.N + q0) * g.r);
        uint32_t qx[16], qa[16], qb2[DQK == 64 ? 16 : 1];
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = p * 4 + sub;
            const uint32_t off = __umul24((uint32_t)tok[q0 + row], fx.c.tsb) + (uint32_t)(hd * g.d + 2 * pair) * 2u;
            qx[p] = *(const uint32_t *)(qbase + off);
            const uint32_t frow = (uint32_t)row * (uint32_t)(g.r * 2);
            qa[p] = *(const uint32_t *)(fqb + frow + 4 * f0);
            if (DQK == 64) qb2[p] = *(const uint32_t *)(fqb + frow + 4 * f1);
        }
        bf16_t *Qs = tiles + wave * 64 * KSTR;
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = p * 4 + sub;
            *(uint32_t *)(Qs + row * KSTR + 2 * pair) = pack_bf16(lo_bf16(qx[p]) * sc, hi_bf16(qx[p]) * sc);
            *(uint32_t *)(Qs + row * KSTR + g.d + 2 * f0) = pack_bf16(lo_bf16(qa[p]) * sp, hi_bf16(qa[p]) * sp);
            if (DQK == 64)
                *(uint32_t *)(Qs + row * KSTR + g.d + 2 * f1) = pack_bf16(lo_bf16(qb2[p]) * sp, hi_bf16(qb2[p]) * sp);
        }
        __syncthreads();
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int t = 0; t < KS; ++t) Q[qb][t] = *(const bf16x8 *)(Qs + (qb * 32 + col) * KSTR + 16 * t + 8 * hf);
        __syncthreads();
    }

    f32x16 O[2];
    float mrun[2] = {0.f, 0.f}, lsum[2];
    bool redo = force_max != 0;
    if (!redo) {
        init_fast_tiles<DQK, NT, ONES>(g, Kf, Vf);
        attend_fast<DQK, ONES, WAVES>(g, fx, rg, tok, Kf, Vf, Q, O, lsum);
        bool bad = false;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float l = ONES ? ones_row(O[qb], g.d) : lsum[qb] + __shfl_xor(lsum[qb], 32);
            if (!((l >= 0x1p-60f) && (l <= 0x1p60f))) bad = true;
        }
        redo = __syncthreads_or(bad);
    }
    if (redo) {
        bf16_t(*Ka)[kTK * KSTR] = (bf16_t(*)[kTK * KSTR]) tiles;
        bf16_t(*Vt)[32 * kVStr] = (bf16_t(*)[32 * kVStr])(tiles + Sm::GEN_K);
        int foff[St::FP];
#pragma unroll
        for (int p = 0; p < St::FP; ++p) {
            int e = p * NT + tid, hr = g.r >> 1;
            int tk = e / hr;
            foff[p] = tk * KSTR + g.d + 2 * (e - tk * hr);
        }
        __syncthreads();
        init_generic_tiles<DQK, NT, ONES>(g, Ka[0], Vt[0]);
        __syncthreads();
        attend<DQK, WAVES, ONES, true>(g, hd, tok, Ka, Vt, foff, Q, k, v, fk, O, mrun, lsum);
    }

    // Normalise, then send O through LDS so that the global stores are token rows: in the
    // accumulator layout a lane holds 16 channels of ONE token, and storing from there would
    // touch 32 token rows per instruction.  Each wave transposes its own 64 x d block in a
    // private LDS area ([64 tokens][34 bf16]: the odd dword stride keeps both sides
    // conflict-free) and writes it out with 16 lanes per token.
    constexpr int ORS = 34;
    // (gated epilogue: the gate words of the rows this lane will store are requested now, so
    // that their latency hides behind the normalisation and the transpose)
    const int sub = lane >> 4, j = lane & 15, jc = 2 * j < g.d ? j : 0;
    uint32_t gw[16];
    if (g.gate != nullptr) {
#pragma unroll
        for (int p = 0; p < 16; ++p)
            gw[p] = *(const uint32_t *)((const bf16_t *)g.gate + (int64_t)tok[q0 + p * 4 + sub] * g.C + hd * g.d + 2 * jc);
    }
    __syncthreads();                                   // every wave is done with the K/V tiles
    bf16_t *Os = tiles + wave * 64 * ORS;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float l = ONES ? ones_row(O[qb], g.d) : lsum[qb] + __shfl_xor(lsum[qb], 32);
        const int n = q0 + qb * 32 + col;
        const float inv = 1.f / l;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            int dv = 8 * (i >> 2) + 4 * hf + (i & 3);
            *(uint32_t *)(Os + (qb * 32 + col) * ORS + dv) = pack_bf16(O[qb][i] * inv, O[qb][i + 1] * inv);
        }
        if (lse != nullptr && hf == 0)
            lse[u * g.N + n] = (mrun[qb] + __builtin_amdgcn_logf(l) + (redo ? 0.f : kTruncLog2)) * kLn2;
    }
    __syncthreads();
    if (2 * j < g.d) {
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const int row = p * 4 + sub;
            const uint32_t w2 = *(const uint32_t *)(Os + row * ORS + 2 * j);
            const int64_t off = (int64_t)tok[q0 + row] * g.C + hd * g.d + 2 * j;
            if (g.gate == nullptr) {
                *(uint32_t *)(out + off) = w2;
            } else {    // CLA gate (Eq. 9) on the way out, the raw O beside it if asked for
                *(uint32_t *)(out + off) = pack_bf16(lo_bf16(w2) * lo_bf16(gw[p]), hi_bf16(w2) * hi_bf16(gw[p]));
                if (g.out_raw) *(uint32_t *)((bf16_t *)g.out_raw + off) = w2;
            }
        }
    }
}

// WAVES = 0: the general kernel (4 waves, 64-key tiles); 4 or 8: the fast kernel.
template <int DQK, bool ONES, int WAVES>
hipError_t launch(const Geo &g, int force_max, const void *q, const void *k, const void *v, const void *fq,
                  const void *fk, void *out, float *lse, hipStream_t st)
{
    constexpr bool FAST = WAVES != 0;
    constexpr int NW = FAST ? WAVES : 4;
    const int nqblk = (g.N + NW * 64 - 1) / (NW * 64);
    const int ntiles = (g.N + kTK - 1) / kTK;
    const size_t dyn = FwdSmem<DQK, FAST, NW>::TILE_BYTES + (FAST ? (size_t)2 * g.M : (size_t)ntiles * kTK) * sizeof(int);
    if (dyn > (size_t)kMaxDynLds) return hipErrorInvalidValue;
    void (*kern)(Geo, int, int, const bf16_t *, const bf16_t *, const bf16_t *, const bf16_t *, const bf16_t *, bf16_t *,
                 float *);
    if constexpr (FAST) kern = mfma_fwd_fast_kernel<DQK, ONES, NW>;
    else kern = mfma_fwd_kernel<DQK, 4, ONES, false>;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [kern] {
        attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynLds);
    });
    if (attr_err != hipSuccess) return attr_err;
    hipLaunchKernelGGL(kern, dim3((unsigned)(g.units * nqblk)), dim3(NW * 64), dyn, st, g, nqblk, force_max,
                       (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v, (const bf16_t *)fq,
                       (const bf16_t *)fk, (bf16_t *)out, lse);
    return hipGetLastError();
}

template <int DQK, bool ONES>
hipError_t launch_pick(const Geo &g, int waves, int force_max, const void *q, const void *k, const void *v,
                       const void *fq, const void *fk, void *out, float *lse, hipStream_t st)
{
    if (waves == 8) return launch<DQK, ONES, 8>(g, force_max, q, k, v, fq, fk, out, lse, st);
    if (waves == 4) return launch<DQK, ONES, 4>(g, force_max, q, k, v, fq, fk, out, lse, st);
    return launch<DQK, ONES, 0>(g, force_max, q, k, v, fq, fk, out, lse, st);
}

}  // namespace

bool mfma_fwd_supported(const Geo &g, int dtype)
{
    return dtype == RIB_BF16 && !(g.flags & RIB_FLAG_VECTOR_ONLY) && g.d <= 32 && (g.d & 1) == 0 && (g.r & 1) == 0 &&
           g.d + g.r <= 64 && g.N >= 64 && g.N <= 9216 && (g.tstride & 1) == 0;
}

// The pipelined fast path needs whole tiles (128 keys with 4 waves, 256 with 8) and 32-bit byte
// offsets built with a 24-bit multiply.  Returns the number of waves to run it with, 0 for the
// general kernel.  Eight waves (each wave then stages half as much per key block) pay off for large
// windows with enough workgroups to go round; at N = 1024 the one workgroup per CU they imply
// leaves the per-workgroup prologue and epilogue uncovered.
static int fast_waves(const Geo &g)
{
    const int64_t tokens = (int64_t)g.B * g.H * g.W;
    const bool small_r = (g.d + g.r <= 48) ? (g.r <= 32) : true;
    if (!(g.r >= 4 && g.d >= 4 && g.N % 128 == 0 && tokens < (1 << 24) && g.tstride * 2 < (1 << 24) &&
          tokens * g.tstride * 2 < ((int64_t)1 << 32) && small_r))
        return 0;
    const bool wide = (g.flags & RIB_FLAG_WIDE) != 0 || (g.N >= 4096 && g.units * (g.N / 512) >= 1024);
    return (wide && g.N % 512 == 0) ? 8 : 4;
}

hipError_t launch_mfma_fwd(const Geo &g, int force_max, const void *q, const void *k, const void *v, const void *fq,
                           const void *fk, void *out, float *lse, hipStream_t st)
{
    const bool ones = g.d < 32;
    const int fast = fast_waves(g);
    if (g.d + g.r <= 48)
        return ones ? launch_pick<48, true>(g, fast, force_max, q, k, v, fq, fk, out, lse, st)
                    : launch_pick<48, false>(g, fast, force_max, q, k, v, fq, fk, out, lse, st);
    return ones ? launch_pick<64, true>(g, fast, force_max, q, k, v, fq, fk, out, lse, st)
                : launch_pick<64, false>(g, fast, force_max, q, k, v, fq, fk, out, lse, st);
}

}  // namespace rib
