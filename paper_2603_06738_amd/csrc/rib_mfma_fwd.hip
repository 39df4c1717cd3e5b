// RIB window attention, forward, on the gfx950 matrix cores (bf16 MFMA, fp32
// accumulation).  Operator: include/rib_attn.h (paper Sec. 2.2; Sec. 3.1 Eq. 5-6).
//
// Shape of the computation
//   A wave owns 64 consecutive window-local queries of one (window, head) unit; a
//   workgroup (4 or 8 waves) owns one (unit, query block) item at a time.  The unit's
//   keys/values stream through LDS in tiles (double buffered), gathered from the
//   channel-last grid through a per-window token map that encodes the window partition
//   and the cyclic shift.  K_aug = [k || f_k] rows are assembled in LDS (Eq. 5), the
//   matching Q_aug = [scale_c q || scale_p f_q] rows (pre-multiplied by log2 e) live in
//   registers; neither ever reaches HBM.  Two kernels: the general one (one workgroup
//   per item, 64-key tiles, any window size) and the streaming one (whole 128/256-key
//   tiles; a grid of resident workgroups, each walking a list of items with one
//   software pipeline running across them).
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
//   term and makes flushed terms negligible).  An item with a failing row (every
//   item, if the caller asks for it) is done again with a running maximum that is
//   raised lazily (only when a tile exceeds it by 2^8) and is subtracted for free
//   as the C operand of the score MFMA; the streaming kernel notes such items and
//   redoes them after its last one.  Both paths compute the exact softmax up to
//   rounding.

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
// The thread id as a value the optimiser cannot trace back to threadIdx.x: lane constants derived
// from it are recomputed where they are used (a few integer instructions) instead of being held
// in registers -- or spilled -- across the MFMA loop.
__device__ __forceinline__ int opaque_tid()
{
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}
__device__ __forceinline__ bf16x8 as_bf16x8(const uint4 &w) { return __builtin_bit_cast(bf16x8, w); }
// Mean relative loss of truncating to bf16 (spacing 2^-7, mantissa log-uniform in [1,2)):
// 2^-8 * 0.7213.  As a log2 it is added to every logit before the truncation (a padding column
// of Q_aug against ones in K_aug) or, where no column is free, to the denominator's log.
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

// Two dwords at a 4-byte aligned address (global memory only needs dword alignment for
// multi-dword accesses; LDS gets them as a two-dword write).
struct __attribute__((packed, aligned(4))) dword2 {
    uint32_t x, y;
};

// Staging registers of one tile: 8 lanes share a token and each thread serves 4 consecutive
// tokens, with 8 bytes per tensor per token.  In LDS a K_aug row of the pipelined path is
// [f_k || k || padding] (RIB part first).
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
__device__ __forceinline__ FastConst<DQK> fast_const(const Geo &g, int hd, int tid)
{
    constexpr int KSTR = DQK + 8, kFVS = FastTile<WAVES>::FVS;
    FastConst<DQK> c;
    const int grp = tid >> 3, j = tid & 7;
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
    c.k_dst = grp * 4 * KSTR + g.r + 2 * dj;
    c.f_dst0 = grp * 4 * KSTR + 2 * f0;
    c.f_dst1 = grp * 4 * KSTR + 2 * f1;
    // V^T rows 2dj .. 2dj+3; the 4 tokens of this lane sit at permuted columns pc .. pc+3
    const int nl = grp * 4;
    const int pc = (nl & ~15) | (((nl >> 2) & 1) << 3) | (((nl >> 3) & 1) << 2);
    c.v_dst = (2 * dj) * kFVS + pc;
    return c;
}

// Byte offsets (from the tensor base) of this lane's piece of its four tokens of the tile that
// starts at window-local token n0.
template <int DQK>
__device__ __forceinline__ void fast_offsets(uint32_t (&off)[4], const FastConst<DQK> &c, const TokMap &tok, int n0)
{
    int t[4];
    tok.quad(n0 + c.tok_idx, t);
#pragma unroll
    for (int p = 0; p < 4; ++p) off[p] = __umul24((uint32_t)t[p], c.tsb) + c.lane_c;
}
// global loads of token p: K and RIB pieces / V piece
template <int DQK>
__device__ __forceinline__ void fast_load_k(FastRegs<DQK> &rg, const FastConst<DQK> &c, const Geo &g, int p, uint32_t off,
                                            const char *kb, const char *fb)
{
    rg.kx[p] = *(const dword2 *)(kb + off);
    const uint32_t row = (uint32_t)(c.tok_idx + p) * (uint32_t)(g.r * 2);
    rg.fa[p] = *(const dword2 *)(fb + row + c.f_off0);
    if (DQK == 64) rg.fb[p] = *(const dword2 *)(fb + row + c.f_off1);
}
template <int DQK>
__device__ __forceinline__ void fast_load_v(FastRegs<DQK> &rg, int p, uint32_t off, const char *vb)
{
    rg.vx[p] = *(const dword2 *)(vb + off);
}
template <int DQK>
__device__ __forceinline__ void fast_load(FastRegs<DQK> &rg, const FastConst<DQK> &c, const Geo &g, const TokMap &tok, int n0,
                                          const char *kb, const char *vb, const char *fb)
{
    uint32_t off[4];
    fast_offsets<DQK>(off, c, tok, n0);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        fast_load_k<DQK>(rg, c, g, p, off[p], kb, fb);
        fast_load_v<DQK>(rg, p, off[p], vb);
    }
}

// LDS writes of token p: its pieces of the K_aug row
template <int DQK>
__device__ __forceinline__ void fast_store_k(const FastRegs<DQK> &rg, const FastConst<DQK> &c, int p, bf16_t *Kf)
{
    constexpr int KSTR = DQK + 8;
    *(dword2 *)(Kf + c.k_dst + p * KSTR) = rg.kx[p];
    *(dword2 *)(Kf + c.f_dst0 + p * KSTR) = rg.fa[p];
    if (DQK == 64) *(dword2 *)(Kf + c.f_dst1 + p * KSTR) = rg.fb[p];
}
// LDS writes of V: half h (0, 1) of this lane's four V^T rows, 4 keys per 8-byte write
template <int DQK, int WAVES>
__device__ __forceinline__ void fast_store_v(const FastRegs<DQK> &rg, const FastConst<DQK> &c, int h, bf16_t *Vf)
{
    constexpr int kFVS = FastTile<WAVES>::FVS;
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
template <int DQK, int WAVES>
__device__ __forceinline__ void fast_store(const FastRegs<DQK> &rg, const FastConst<DQK> &c, bf16_t *Kf, bf16_t *Vf)
{
#pragma unroll
    for (int p = 0; p < 4; ++p) fast_store_k<DQK>(rg, c, p, Kf);
    fast_store_v<DQK, WAVES>(rg, c, 0, Vf);
    fast_store_v<DQK, WAVES>(rg, c, 1, Vf);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
#define kOnes2 __builtin_bit_cast(bf16x2, 0x3f803f80u)

// Where the staging of a streaming workgroup reads next: the load cursor runs two tiles ahead
// of the arithmetic and crosses from one (unit, query block) item into the next on its own.
struct LoadCursor {
    TokMap tok;                     // window map of the cursor's item
    const char *fbase;              // RIB table of the cursor's head
    int hd;                         // the cursor's head
    int tile;                       // tile the next request fetches
};

// A operands of two consecutive key blocks (double buffer); they live across tiles.
template <int DQK>
struct Operands {
    bf16x8 k[2][DQK / 16], v[2][2];
};
template <int DQK, int WAVES>
__device__ __forceinline__ void read_k_operand(Operands<DQK> &A, int buf, const bf16_t *Kc, int kb)
{
    constexpr int KSTR = DQK + 8;
    const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int t = 0; t < DQK / 16; ++t) A.k[buf][t] = *(const bf16x8 *)(Kc + (kb * 32 + col) * KSTR + 16 * t + 8 * hf);
}
template <int DQK, int WAVES>
__device__ __forceinline__ void read_v_operand(Operands<DQK> &A, int buf, const bf16_t *Vc, int kb)
{
    constexpr int kFVS = FastTile<WAVES>::FVS;
    const int lane = threadIdx.x & 63, col = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int t = 0; t < 2; ++t) A.v[buf][t] = *(const bf16x8 *)(Vc + col * kFVS + kb * 32 + 16 * t + 8 * hf);
}

// One K/V tile of the pipelined path: the wave's 64 queries against the kFT keys staged at
// (Kc, Vc).  The instruction order is written out and pinned with scheduling fences.  For the
// 32x32 block s of the tile the wave issues, interleaved,
//   the score MFMAs of block s+1, the 16 exp2 + 8 bf16 packs of block s, the 2 PV MFMAs of block s-1,
// so that the matrix pipe and the vector ALU always have independent work.  Staging rides in the
// same stream: the tile requested one tile ago (`rg`) is written to (Kn, Vn) during the first
// steps and the cursor's tile is requested into the registers just freed.  The A operands of a
// key block are read from LDS two steps before their first use.  The workgroup barrier sits
// BEFORE the last two steps, right after the tile's last LDS access, and the first operands of
// the next tile (which lives in (Kn, Vn)) are read behind it: the tail of this tile's arithmetic
// covers the barrier and the read latency.  On entry A holds the operands of key blocks 0 and 1
// (V: block 0) of this tile; on exit those of the next tile.
template <int DQK, bool ONES, int WAVES>
__device__ __forceinline__ void fast_tile(const Geo &g, const LoadCursor &lc, const char *kbase, const char *vbase,
                                          FastRegs<DQK> &rg, Operands<DQK> &A, const bf16_t *Kc, const bf16_t *Vc, bf16_t *Kn,
                                          bf16_t *Vn, const bf16x8 (&Q)[2][DQK / 16], f32x16 (&O)[2], float (&lsum)[2])
{
    constexpr int KS = DQK / 16;
    constexpr int kFT = FastTile<WAVES>::FT;
    constexpr int NKB = kFT / 32, NSTEP = 2 * NKB;        // key blocks per tile; (key block, query block) steps
    static_assert(NKB >= 4, "the staging schedule below uses steps 0..7");
    const f32x16 zero = {0};
    const char *fsrc = lc.fbase + (uint32_t)lc.tile * ((uint32_t)kFT * (uint32_t)(g.r * 2));

    f32x16 S[2];
    uint4 P[2][2];                  // packed bf16 probabilities: B operands of the PV MFMAs
    uint32_t off[4];                // where the cursor's tile lies in memory (this lane's pieces)
    const FastConst<DQK> c = fast_const<DQK, WAVES>(g, lc.hd, opaque_tid());
    S[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.k[0][0], Q[0][0], zero, 0, 0, 0);
#pragma unroll
    for (int t = 1; t < KS; ++t) S[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.k[0][t], Q[0][t], S[0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);

#pragma unroll
    for (int s = 0; s < NSTEP; ++s) {
        const int kb = s >> 1, qb = s & 1, cs = s & 1, ns = cs ^ 1;
        const int s1 = s + 1, kb1 = s1 >> 1, qb1 = s1 & 1;
        const int kbp = (s - 1) >> 1, qbp = (s - 1) & 1;
        float pe[16];
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            // one MFMA: scores of the next block (groups 0..2) / first PV product of the previous block
            if (grp < 3) {
                if (s < NSTEP - 1 && grp < 2) {
                    S[ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.k[kb1 & 1][grp], Q[qb1][grp], grp == 0 ? zero : S[ns], 0,
                                                                     0, 0);
                }
                if (s < NSTEP - 1 && grp == 2) {
#pragma unroll
                    for (int t = 2; t < KS; ++t)
                        S[ns] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.k[kb1 & 1][t], Q[qb1][t], S[ns], 0, 0, 0);
                }
            } else if (s > 0) {
                O[qbp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.v[kbp & 1][0], as_bf16x8(P[ns][0]), O[qbp], 0, 0, 0);
            }
            // 4 exp2 and 2 packs of this block
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
            // ---- this group's share of the staging ----
            if (s < 4) {                // steps 0..3: K and RIB pieces of token s out, the cursor's in
                if (grp == 0) fast_store_k<DQK>(rg, c, s, Kn);
                if (grp == 0 && s == 0) fast_offsets<DQK>(off, c, lc.tok, lc.tile * kFT);
                if (grp == 2) fast_load_k<DQK>(rg, c, g, s, off[s], kbase, fsrc);
            } else if (s < 6) {         // steps 4, 5: V^T rows out
                if (grp == 0) fast_store_v<DQK, WAVES>(rg, c, s - 4, Vn);
            } else if (s < 8) {         // steps 6, 7: the cursor's V pieces in
                if (grp == 0 || grp == 2) {
                    const int p = 2 * (s - 6) + (grp >> 1);
                    fast_load_v<DQK>(rg, p, off[p], vbase);
                }
            }
            // ---- operand reads: at odd steps, K of key block kb+2 and V of key block kb+1; behind
            // the barrier (the last two steps) the next tile's first blocks ----
            if (qb == 1 && grp == 1) {
                if (kb + 2 < NKB) read_k_operand<DQK, WAVES>(A, kb & 1, Kc, kb + 2);
                else if (s == NSTEP - 1) read_k_operand<DQK, WAVES>(A, 1, Kn, 1);
            }
            if (qb == 1 && grp == 3) {
                if (kb + 1 < NKB) read_v_operand<DQK, WAVES>(A, (kb + 1) & 1, Vc, kb + 1);
                else read_v_operand<DQK, WAVES>(A, 0, Vn, 0);
            }
            if (s == NSTEP - 2 && grp == 1) read_k_operand<DQK, WAVES>(A, 0, Kn, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // second PV MFMA of the previous block
        if (s > 0) O[qbp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.v[kbp & 1][1], as_bf16x8(P[ns][1]), O[qbp], 0, 0, 0);
        if (s == NSTEP - 3) {           // the tile's last LDS access is behind us
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // drain: PV of the last block
    O[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.v[(NKB - 1) & 1][0], as_bf16x8(P[1][0]), O[1], 0, 0, 0);
    O[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A.v[(NKB - 1) & 1][1], as_bf16x8(P[1][1]), O[1], 0, 0, 0);
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
// `bias`: the first padding column of K_aug holds 1.0 (its partner in Q_aug is a constant that
// the score MFMA then adds to every logit), the others 0.
template <int DQK, int NT, bool ONES>
__device__ __forceinline__ void init_fast_tiles(const Geo &g, bf16_t *Kf, bf16_t *Vf, bool bias)
{
    constexpr int KSTR = DQK + 8, kFT = FastTile<NT / 64>::FT, kFVS = FastTile<NT / 64>::FVS;
    const int pad0 = g.d + g.r;                                  // even; columns pad0..DQK-1 are constant
    for (int row = threadIdx.x; row < 2 * kFT; row += NT)
        for (int c = pad0; c < DQK; c += 2) *(uint32_t *)(Kf + row * KSTR + c) = (bias && c == pad0) ? 0x00003f80u : 0u;
    const int vrows = 32 - g.d;                                  // rows d..31 of both stages
    for (int e = threadIdx.x; e < 2 * vrows * (kFVS / 2); e += NT) {
        const int per = vrows * (kFVS / 2);
        const int st = e / per, rem = e - st * per;
        const int row = g.d + rem / (kFVS / 2), cw = rem - (rem / (kFVS / 2)) * (kFVS / 2);
        *(uint32_t *)(Vf + (st * 32 + row) * kFVS + 2 * cw) = (ONES && row == g.d) ? 0x3f803f80u : 0u;
    }
}

constexpr int kMaxItemsPerWg = 512;    // items one workgroup of the streaming kernel may be given per launch

template <int DQK, bool FAST, int WAVES = 4>
struct FwdSmem {
    static constexpr int KSTR = DQK + 8;
    static constexpr int GEN_K = 2 * kTK * KSTR, GEN_V = 2 * 32 * kVStr;       // bf16 elements
    static constexpr int FAST_K = 2 * FastTile<WAVES>::FT * KSTR, FAST_V = 2 * 32 * FastTile<WAVES>::FVS;
    static constexpr int TILE_ELEMS = FAST ? (FAST_K + FAST_V) : (GEN_K + GEN_V);
    static constexpr size_t TILE_BYTES = (size_t)TILE_ELEMS * sizeof(bf16_t);
    // streaming kernel: per-wave area for Q staging ([32][KSTR]) and the output transpose ([32][34])
    static constexpr int WAVE_ELEMS = 32 * KSTR;
    // ... followed by the redo flags [kMaxItemsPerWg] and three window maps of 2M integers
    static __device__ __forceinline__ int *redo_flags(char *smem)
    {
        return (int *)(smem + TILE_BYTES + (size_t)WAVES * WAVE_ELEMS * sizeof(bf16_t));
    }
    static_assert(!FAST || TILE_ELEMS >= GEN_K + GEN_V, "the general path borrows the pipelined path's tiles");
};

// One (unit, query block) item on the general path: Q_aug rows staged through LDS one wave at a
// time, the optimistic pass unless ALWAYS_MAX (or force_max), the max-tracking pass if needed,
// then normalisation and the scatter straight from the accumulator layout.  `tok` maps
// window-local tokens to grid tokens (a table with -1 past N, or a TokMap when N is whole
// tiles); `tiles` is LDS for FwdSmem<DQK, false>::TILE_BYTES.  Ends with every wave past its
// last LDS access only after the caller's next barrier.
template <int DQK, int WAVES, bool ONES, bool ALWAYS_MAX, class TK>
__device__ __forceinline__ void generic_item(const Geo &g, int64_t u, int blk, int hd, const TK &tok, bf16_t *tiles,
                                             int force_max, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                             const bf16_t *__restrict__ v, const bf16_t *__restrict__ fq,
                                             const bf16_t *__restrict__ fk, bf16_t *__restrict__ out,
                                             float *__restrict__ lse)
{
    constexpr int NT = WAVES * 64;
    constexpr int KS = DQK / 16;
    constexpr int KSTR = DQK + 8;
    using St = Stage<DQK, WAVES>;
    using Sm = FwdSmem<DQK, false>;
    bf16_t(*Ka)[kTK * KSTR] = (bf16_t(*)[kTK * KSTR]) tiles;
    bf16_t(*Vt)[32 * kVStr] = (bf16_t(*)[32 * kVStr])(tiles + Sm::GEN_K);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, hf = lane >> 5;
    const int ntiles = (g.N + kTK - 1) / kTK;

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
    bool redo = ALWAYS_MAX || force_max != 0;
    if constexpr (!ALWAYS_MAX) {
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

template <int DQK, int WAVES, bool ONES, bool FAST>
__global__ __launch_bounds__(WAVES * 64, 2) void mfma_fwd_kernel(
    Geo g, int nqblk, int force_max, const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
    const bf16_t *__restrict__ v, const bf16_t *__restrict__ fq, const bf16_t *__restrict__ fk,
    bf16_t *__restrict__ out, float *__restrict__ lse)
{
    constexpr int NT = WAVES * 64;
    using Sm = FwdSmem<DQK, FAST>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int *tok = (int *)(smem + Sm::TILE_BYTES);   // [ntiles*64] grid token of each window-local token, -1 past N

    // Workgroups are dealt round-robin to the 8 XCDs; renumber them so that each XCD
    // works on a contiguous range of (unit, query block) and its L2 sees all users
    // of a window's K/V lines.
    const int G = gridDim.x, per = G >> 3, rem = G & 7, xcd = blockIdx.x & 7;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    const int64_t u = logical / nqblk;
    const int blk = logical - (int)(u * nqblk);
    const int w = (int)(u / g.heads), hd = (int)(u - (int64_t)w * g.heads);
    const int ntiles = (g.N + kTK - 1) / kTK;
    fill_tok_table<NT>(g, w, tok, ntiles * kTK);
    generic_item<DQK, WAVES, ONES, false>(g, u, blk, hd, tok, (bf16_t *)smem, force_max, q, k, v, fq, fk, out, lse);
}

// ---------------------------------------------------------------------------------------
// Streaming forward kernel for the common case (whole 128-key tiles, 32-bit byte offsets,
// r > 0).  The grid is as many workgroups as the chip holds at once; each walks a list of
// (unit, query block) items and keeps ONE software pipeline running across them: while the
// last K/V tiles of an item are in the matrix cores, the first tiles of the next item are
// already being staged (the load cursor crosses item boundaries on its own), so only the
// very first item of a workgroup waits for memory.  Between two items a wave normalises and
// stores its 64 output rows and stages its next 64 Q_aug rows through a wave-private LDS
// area; no workgroup barrier is involved, the other waves carry on with the next item.
//
// Items are dealt so that the workgroups of one XCD work on neighbouring items at the same
// time (workgroup j of the XCD's nx takes items first + j, first + j + nx, ...): the users of
// a window's K/V lines then meet in that XCD's L2.
//
// Items in which a wave finds a row whose softmax denominator left the safe range are noted in
// LDS and redone on the max-tracking general path after the workgroup's last item (cold code: placed there it
// shares no live registers with the loop and does not disturb the pipeline).
struct Item {
    int u, blk, w, hd;
};
__device__ __forceinline__ Item decode_item(const Geo &g, int item, int nqblk)
{
    Item it;
    it.u = item / nqblk;
    it.blk = item - it.u * nqblk;
    it.w = it.u / g.heads;
    it.hd = it.u - it.w * g.heads;
    return it;
}
__device__ __forceinline__ TokMap map_at(const Geo &g, const int *slot)
{
    TokMap m;
    m.rowb = slot;
    m.colo = slot + g.M;
    m.inv_m = g.inv_m;
    m.M = g.M;
    return m;
}



// Raw q / f_q words of a wave's 64 query rows, between their request and their staging.  Two layouts
// share the registers: the general one (16 lanes per token, 4 tokens per pass: w[p] content pair, w[16 + p]
// and w[32 + p] RIB pairs of row p*4 + sub) and the direct one (the lane's own two query columns in operand
// order: w[(qb * KS + t) * 4 + i] = dword i of k-step t).
template <int DQK>
struct QRaw {
    uint32_t w[DQK == 64 ? 48 : 32];
};
template <int DQK>
__device__ __forceinline__ void q_request(QRaw<DQK> &r, const Geo &g, const TokMap &tok, int hd, int q0, uint32_t tsb,
                                          const bf16_t *__restrict__ q, const bf16_t *__restrict__ fq)
{
    const int lane = opaque_tid() & 63, sub = lane >> 4, j = lane & 15, hp = g.d >> 1, rh = g.r >> 1;
    const int pair = j < hp ? j : hp - 1;
    const int f0 = j < rh ? j : rh - 1, f1 = 16 + j < rh ? 16 + j : rh - 1;
    const char *qbase = (const char *)q;
    const char *fqb = (const char *)(fq + ((int64_t)hd * g.N + q0) * g.r);
#pragma unroll
    for (int p = 0; p < 16; ++p) {
        const int row = p * 4 + sub;
        const uint32_t off = __umul24((uint32_t)tok[q0 + row], tsb) + (uint32_t)(hd * g.d + 2 * pair) * 2u;
        r.w[p] = *(const uint32_t *)(qbase + off);
        const uint32_t frow = (uint32_t)row * (uint32_t)(g.r * 2);
        r.w[16 + p] = *(const uint32_t *)(fqb + frow + 4 * f0);
        if (DQK == 64) r.w[32 + p] = *(const uint32_t *)(fqb + frow + 4 * f1);
    }
}
// Scale (Eq. 5, times log2 e), round to bf16 and turn the rows into the B operands of the score
// MFMA, 32 rows at a time through the wave's own LDS area `Ws` ([32][DQK + 8] bf16).  `padw` is
// the word written to the first padding column pair (the logit offset, or 0).
template <int DQK>
__device__ __forceinline__ void q_stage(const QRaw<DQK> &r, const Geo &g, bf16_t *Ws, uint32_t padw,
                                        bf16x8 (&Q)[2][DQK / 16])
{
    constexpr int KS = DQK / 16, KSTR = DQK + 8;
    const int lane = opaque_tid() & 63, sub = lane >> 4, j = lane & 15, hp = g.d >> 1, rh = g.r >> 1;
    const int col = lane & 31, hf = lane >> 5;
    const int pair = j < hp ? j : hp - 1;
    const int f0 = j < rh ? j : rh - 1, f1 = 16 + j < rh ? 16 + j : rh - 1;
    const float sc = g.scale_c * kLog2e, sp = g.scale_p * kLog2e;
#pragma unroll
    for (int ps = 0; ps < 2; ++ps) {
        if (hf == 0)
            for (int c = g.d + g.r; c < DQK; c += 2) *(uint32_t *)(Ws + col * KSTR + c) = (c == g.d + g.r) ? padw : 0u;
#pragma unroll
        for (int pp = 0; pp < 8; ++pp) {
            const int p = ps * 8 + pp, row = pp * 4 + sub;
            // (column order of the pipelined path: RIB part first, as in its K_aug rows)
            *(uint32_t *)(Ws + row * KSTR + g.r + 2 * pair) = pack_bf16(lo_bf16(r.w[p]) * sc, hi_bf16(r.w[p]) * sc);
            *(uint32_t *)(Ws + row * KSTR + 2 * f0) = pack_bf16(lo_bf16(r.w[16 + p]) * sp, hi_bf16(r.w[16 + p]) * sp);
            if (DQK == 64)
                *(uint32_t *)(Ws + row * KSTR + 2 * f1) = pack_bf16(lo_bf16(r.w[32 + p]) * sp, hi_bf16(r.w[32 + p]) * sp);
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t = 0; t < KS; ++t) Q[ps][t] = *(const bf16x8 *)(Ws + col * KSTR + 16 * t + 8 * hf);
        __builtin_amdgcn_wave_barrier();
    }
}

// The direct form, for ranks that are multiples of 8: the row [f_q || q || padding] then falls into whole
// 16-byte pieces of ONE source each, and a lane fetches the pieces of its own two query columns in
// operand order -- piece 2t + hf of row q0 + 32 qb + col is k-step t of query block qb -- with no trip
// through LDS: 3 or 4 loads per query block instead of 16 or 24, one token look-up instead of eight.
// The last content piece may be short (d = 30: 12 bytes); nothing past the head's slice is read.
struct __attribute__((packed, aligned(4))) dword4 {
    uint32_t x, y, z, w;
};
template <int DQK>
__device__ __forceinline__ void q_request_direct(QRaw<DQK> &r, const Geo &g, const TokMap &tok, int hd, int q0,
                                                 uint32_t tsb, const bf16_t *__restrict__ q,
                                                 const bf16_t *__restrict__ fq)
{
    constexpr int KS = DQK / 16;
    const int lane = opaque_tid() & 63, col = lane & 31, hf = lane >> 5;
    const int nf = g.r >> 3;                                    // RIB pieces
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int n = q0 + qb * 32 + col;
        const char *qsrc = (const char *)q + (__umul24((uint32_t)tok[n], tsb) + (uint32_t)(hd * g.d) * 2u);
        const char *fsrc = (const char *)fq + (uint32_t)(hd * g.N + n) * (uint32_t)(g.r * 2);
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const int p = 2 * t + hf, base = (qb * KS + t) * 4;
            r.w[base] = r.w[base + 1] = r.w[base + 2] = r.w[base + 3] = 0u;
            if (p < nf) {
                const dword4 x = *(const dword4 *)(fsrc + 16 * p);
                r.w[base] = x.x, r.w[base + 1] = x.y, r.w[base + 2] = x.z, r.w[base + 3] = x.w;
            } else {
                const int e0 = 8 * (p - nf), nd = (g.d - e0) >> 1;      // first content element, dwords left
                const char *src = qsrc + 2 * e0;
                if (nd >= 4) {
                    const dword4 x = *(const dword4 *)src;
                    r.w[base] = x.x, r.w[base + 1] = x.y, r.w[base + 2] = x.z, r.w[base + 3] = x.w;
                } else {
                    if (nd >= 2) {
                        const dword2 x = *(const dword2 *)src;
                        r.w[base] = x.x, r.w[base + 1] = x.y;
                    }
                    if (nd == 1) r.w[base] = *(const uint32_t *)src;
                    if (nd == 3) r.w[base + 2] = *(const uint32_t *)(src + 8);
                }
            }
        }
    }
}
template <int DQK>
__device__ __forceinline__ void q_stage_direct(const QRaw<DQK> &r, const Geo &g, uint32_t padw, bool bias,
                                               bf16x8 (&Q)[2][DQK / 16])
{
    constexpr int KS = DQK / 16;
    const int hf = (opaque_tid() & 63) >> 5;
    const int nf = g.r >> 3;
    const float sc = g.scale_c * kLog2e, sp = g.scale_p * kLog2e;
    const int eb = g.d + g.r;                                   // the column of the logit offset
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            const int p = 2 * t + hf, base = (qb * KS + t) * 4;
            const float s = p < nf ? sp : sc;
            uint4 o;
            o.x = pack_bf16(lo_bf16(r.w[base]) * s, hi_bf16(r.w[base]) * s);
            o.y = pack_bf16(lo_bf16(r.w[base + 1]) * s, hi_bf16(r.w[base + 1]) * s);
            o.z = pack_bf16(lo_bf16(r.w[base + 2]) * s, hi_bf16(r.w[base + 2]) * s);
            o.w = pack_bf16(lo_bf16(r.w[base + 3]) * s, hi_bf16(r.w[base + 3]) * s);
            if (bias && p == (eb >> 3)) {       // (d and r even, r a multiple of 8: the column opens a dword)
                const int dw = (eb & 7) >> 1;
                o.x = dw == 0 ? padw : o.x, o.y = dw == 1 ? padw : o.y, o.z = dw == 2 ? padw : o.z, o.w = dw == 3 ? padw : o.w;
            }
            Q[qb][t] = __builtin_bit_cast(bf16x8, o);
        }
}

// The pipelined walk of one workgroup over its items (see the kernel below).
template <int DQK, bool ONES, int WAVES>
__device__ __forceinline__ void stream_items(const Geo &g, int nqblk, int item0, int nx, int my_n, char *smem,
                                             const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                             const bf16_t *__restrict__ v, const bf16_t *__restrict__ fq,
                                             const bf16_t *__restrict__ fk, bf16_t *__restrict__ out,
                                             float *__restrict__ lse)
{
    constexpr int NT = WAVES * 64;
    constexpr int kFT = FastTile<WAVES>::FT, kFVS = FastTile<WAVES>::FVS;
    constexpr int KSTR = DQK + 8;
    constexpr int KSZ = kFT * KSTR, VSZ = 32 * kFVS;     // bf16 per stage
    using Sm = FwdSmem<DQK, true, WAVES>;
    bf16_t *tiles = (bf16_t *)smem;
    bf16_t *Kf = tiles, *Vf = tiles + Sm::FAST_K;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    bf16_t *Ws = tiles + Sm::TILE_ELEMS + wave * Sm::WAVE_ELEMS;                  // this wave's own LDS area
    int *redo_flag = Sm::redo_flags(smem);
    int *maps = redo_flag + kMaxItemsPerWg;                                       // 3 window maps
    const int map_words = 2 * g.M;
    const int ntiles = g.N / kFT;

    // Truncating P to bf16 loses half a unit in the last place on average.  Where Q_aug / K_aug
    // have a padding column, a constant log2(1 + 2^-8 * 0.7213) rides there against ones, so that
    // every P is scaled up by that mean loss BEFORE it is truncated: values that are exactly
    // representable (uniform rows, one-hot rows) come through unchanged, the others are right on
    // average, and numerator and denominator still share the same P.  Without a padding column
    // the mean loss is added to the denominator's log2 instead.
    const bool bias = g.d + g.r < DQK;
    const uint32_t padw = bias ? (uint32_t)narrow_bf16(kTruncLog2) : 0u;
    const uint32_t tsb = (uint32_t)g.tstride * 2u;
    // Q rows straight into operand order (see q_request_direct) where that measured faster: the 64-column
    // variants with d = 32 (r = 32: 6 % at N = 2304).  With 48 columns the scattered 16-byte loads take longer to
    // land than the 16-lanes-per-token requests, and the time between items is waiting, not issuing: 2 % slower.
    const bool direct = DQK == 64 && !ONES && (g.r & 7) == 0;
    const char *kbase = (const char *)k, *vbase = (const char *)v;

    Item ci = decode_item(g, item0, nqblk);
    fill_tok_map<NT>(g, ci.w, maps);
    if (my_n > 1) fill_tok_map<NT>(g, decode_item(g, item0 + nx, nqblk).w, maps + map_words);
    init_fast_tiles<DQK, NT, ONES>(g, Kf, Vf, bias);
    __syncthreads();

    LoadCursor lc;
    int lt = 0;                         // item of the load cursor
    lc.hd = ci.hd;
    lc.tok = map_at(g, maps);
    lc.fbase = (const char *)(fk + (int64_t)ci.hd * g.N * g.r);
    lc.tile = 0;
    auto advance = [&]() {
        if (++lc.tile == ntiles) {
            if (lt + 1 < my_n) {
                ++lt;
                const Item li = decode_item(g, item0 + nx * lt, nqblk);
                lc.hd = li.hd;
                lc.tok = map_at(g, maps + (lt % 3) * map_words);
                lc.fbase = (const char *)(fk + (int64_t)li.hd * g.N * g.r);
                lc.tile = 0;
            } else {
                lc.tile = ntiles - 1;   // past the end: the last tile is staged again and never used
            }
        }
    };
    auto request = [&](FastRegs<DQK> &rg) {
        fast_load<DQK>(rg, fast_const<DQK, WAVES>(g, lc.hd, opaque_tid()), g, lc.tok, lc.tile * kFT, kbase, vbase,
                       lc.fbase + (uint32_t)lc.tile * ((uint32_t)kFT * (uint32_t)(g.r * 2)));
    };

    FastRegs<DQK> rg;
    Operands<DQK> A;
    bf16x8 Q[2][DQK / 16];
    {
        request(rg);
        advance();
        QRaw<DQK> qr;
        if (direct) q_request_direct<DQK>(qr, g, lc.tok, ci.hd, ci.blk * NT + wave * 64, tsb, q, fq);   // (cursor still in item 0)
        else q_request<DQK>(qr, g, lc.tok, ci.hd, ci.blk * NT + wave * 64, tsb, q, fq);
        {
            const FastConst<DQK> c0 = fast_const<DQK, WAVES>(g, ci.hd, opaque_tid());
            fast_store<DQK, WAVES>(rg, c0, Kf, Vf);
        }
        request(rg);
        advance();
        if (direct) q_stage_direct<DQK>(qr, g, padw, bias, Q);
        else q_stage<DQK>(qr, g, Ws, padw, Q);
    }
    for (int e = tid; e < my_n; e += NT) redo_flag[e] = 0;
    __syncthreads();
    read_k_operand<DQK, WAVES>(A, 0, Kf, 0);
    read_k_operand<DQK, WAVES>(A, 1, Kf, 1);
    read_v_operand<DQK, WAVES>(A, 0, Vf, 0);

    int cur = 0;
    for (int t = 0; t < my_n; ++t) {
        f32x16 O[2];
        float lsum[2] = {0.f, 0.f};
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[qb][i] = 0.f;

        for (int tile = 0; tile < ntiles; ++tile) {
            // the map of the item after next goes into the slot the previous item has left; the
            // barrier inside the last tile publishes it
            if (tile == ntiles - 1 && t + 2 < my_n)
                fill_tok_map<NT>(g, decode_item(g, item0 + nx * (t + 2), nqblk).w, maps + ((t + 2) % 3) * map_words);
            fast_tile<DQK, ONES, WAVES>(g, lc, kbase, vbase, rg, A, Kf + cur * KSZ, Vf + cur * VSZ, Kf + (cur ^ 1) * KSZ,
                                        Vf + (cur ^ 1) * VSZ, Q, O, lsum);
            advance();
            cur ^= 1;
        }
        // A wave whose rows left the safe range notes the item for the cold path and skips its
        // stores; the other waves' results are simply written again there.
        bool bad = false;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const float l = ONES ? ones_row(O[qb], g.d) : lsum[qb] + __shfl_xor(lsum[qb], 32);
            if (!((l >= 0x1p-60f) && (l <= 0x1p60f))) bad = true;
        }
        const bool redo = __any(bad);
        if (redo) redo_flag[t] = 1;

        const int q0 = ci.blk * NT + wave * 64;
        const TokMap ctok = map_at(g, maps + (t % 3) * map_words);

        QRaw<DQK> qr;
        Item ni = ci;
        if (t + 1 < my_n) {     // the next item's Q rows are requested now and land during the epilogue
            ni = decode_item(g, item0 + nx * (t + 1), nqblk);
            const TokMap ntok = map_at(g, maps + ((t + 1) % 3) * map_words);
            if (direct) q_request_direct<DQK>(qr, g, ntok, ni.hd, ni.blk * NT + wave * 64, tsb, q, fq);
            else q_request<DQK>(qr, g, ntok, ni.hd, ni.blk * NT + wave * 64, tsb, q, fq);
        }

        // Two forms of the output stage; which one is faster was measured per variant: the narrow variants
        // with the ones row (d < 32, d + r <= 48: the benchmark configs, r = 18) store directly (1 % at N = 1024,
        // 5 % at N = 256), the 64-column and d = 32 variants are 1-4 % faster through the LDS transpose.
        constexpr bool kDirectStores = ONES && DQK <= 48;
        if constexpr (kDirectStores) {
        if (!redo) {
            // Normalise and store straight from the accumulator layout: a lane holds, for ONE token, four
            // groups of four consecutive channels (8 bytes each), so a token's head slice leaves as four
            // 8-byte stores of the two lane halves, back to back.  (Sending O through LDS first, for
            // stores of whole token rows, took more instructions than the wider rows saved.)
            const int lane = opaque_tid() & 63, col = lane & 31, hf = lane >> 5;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                // byte offset of this lane's token slice in a dense [tokens][C] tensor (fits 32 bits, as
                // every offset on this path does)
                const uint32_t obase = ((uint32_t)ctok[q0 + qb * 32 + col] * (uint32_t)g.C + (uint32_t)(ci.hd * g.d + 4 * hf)) * 2u;
                dword2 gw[4];
                if (g.gate != nullptr) {    // gate words of the channels this lane will store: requested early
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) {
                        gw[c4].x = 0u, gw[c4].y = 0u;
                        const char *gp = (const char *)g.gate + (obase + 16u * c4);
                        if (8 * c4 + 4 * hf + 4 <= g.d) gw[c4] = *(const dword2 *)gp;
                        else if (8 * c4 + 4 * hf + 2 <= g.d) gw[c4].x = *(const uint32_t *)gp;
                    }
                }
                const float l = ONES ? ones_row(O[qb], g.d) : lsum[qb] + __shfl_xor(lsum[qb], 32);
                const float inv = 1.f / l;
                if (lse != nullptr && hf == 0)
                    lse[(int64_t)ci.u * g.N + q0 + qb * 32 + col] = (__builtin_amdgcn_logf(l) + (bias ? 0.f : kTruncLog2)) * kLn2;
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4) {
                    dword2 w2;
                    w2.x = pack_bf16(O[qb][4 * c4] * inv, O[qb][4 * c4 + 1] * inv);
                    w2.y = pack_bf16(O[qb][4 * c4 + 2] * inv, O[qb][4 * c4 + 3] * inv);
                    dword2 wo = w2;
                    if (g.gate != nullptr) {    // CLA gate (Eq. 9) on the way out, the raw O beside it if asked for
                        wo.x = pack_bf16(lo_bf16(w2.x) * lo_bf16(gw[c4].x), hi_bf16(w2.x) * hi_bf16(gw[c4].x));
                        wo.y = pack_bf16(lo_bf16(w2.y) * lo_bf16(gw[c4].y), hi_bf16(w2.y) * hi_bf16(gw[c4].y));
                    }
                    const uint32_t off = obase + 16u * c4;
                    if (8 * c4 + 4 * hf + 4 <= g.d) {
                        *(dword2 *)((char *)out + off) = wo;
                        if (g.gate != nullptr && g.out_raw) *(dword2 *)((char *)g.out_raw + off) = w2;
                    } else if (8 * c4 + 4 * hf + 2 <= g.d) {
                        *(uint32_t *)((char *)out + off) = wo.x;
                        if (g.gate != nullptr && g.out_raw) *(uint32_t *)((char *)g.out_raw + off) = w2.x;
                    }
                }
            }
        }
        } else {
        if (!redo) {
            // Normalise, then send O through LDS so that the global stores are token rows: in the
            // accumulator layout a lane holds 16 channels of ONE token, and storing from there would
            // touch 32 token rows per instruction.  Each wave transposes 32 x d at a time in its own
            // LDS area ([32 tokens][34 bf16]: the odd dword stride keeps both sides conflict-free)
            // and writes it out with 16 lanes per token.
            constexpr int ORS = 34;
            const int lane = opaque_tid() & 63, col = lane & 31, hf = lane >> 5;
            const int sub = lane >> 4, jj = lane & 15, jc = 2 * jj < g.d ? jj : 0;
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                uint32_t gw[8];
                if (g.gate != nullptr) {    // gate words of the rows this lane will store: requested early
#pragma unroll
                    for (int pp = 0; pp < 8; ++pp)
                        gw[pp] = *(const uint32_t *)((const bf16_t *)g.gate +
                                                     (int64_t)ctok[q0 + qb * 32 + pp * 4 + sub] * g.C + ci.hd * g.d + 2 * jc);
                }
                const float l = ONES ? ones_row(O[qb], g.d) : lsum[qb] + __shfl_xor(lsum[qb], 32);
                const float inv = 1.f / l;
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const int dv = 8 * (i >> 2) + 4 * hf + (i & 3);
                    *(uint32_t *)(Ws + col * ORS + dv) = pack_bf16(O[qb][i] * inv, O[qb][i + 1] * inv);
                }
                if (lse != nullptr && hf == 0)
                    lse[(int64_t)ci.u * g.N + q0 + qb * 32 + col] = (__builtin_amdgcn_logf(l) + (bias ? 0.f : kTruncLog2)) * kLn2;
                __builtin_amdgcn_wave_barrier();
                if (2 * jj < g.d) {
#pragma unroll
                    for (int pp = 0; pp < 8; ++pp) {
                        const int row = pp * 4 + sub;
                        const uint32_t w2 = *(const uint32_t *)(Ws + row * ORS + 2 * jj);
                        const int64_t off = (int64_t)ctok[q0 + qb * 32 + row] * g.C + ci.hd * g.d + 2 * jj;
                        if (g.gate == nullptr) {
                            *(uint32_t *)(out + off) = w2;
                        } else {    // CLA gate (Eq. 9) on the way out, the raw O beside it if asked for
                            *(uint32_t *)(out + off) = pack_bf16(lo_bf16(w2) * lo_bf16(gw[pp]), hi_bf16(w2) * hi_bf16(gw[pp]));
                            if (g.out_raw) *(uint32_t *)((bf16_t *)g.out_raw + off) = w2;
                        }
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
        }

        if (t + 1 < my_n) {
            ci = ni;
            if (direct) q_stage_direct<DQK>(qr, g, padw, bias, Q);
            else q_stage<DQK>(qr, g, Ws, padw, Q);
        }
    }
}

template <int DQK, bool ONES, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 2) void mfma_fwd_stream_kernel(
    Geo g, int nqblk, int item_base, int n_items, int force_max, const bf16_t *__restrict__ q,
    const bf16_t *__restrict__ k, const bf16_t *__restrict__ v, const bf16_t *__restrict__ fq,
    const bf16_t *__restrict__ fk, bf16_t *__restrict__ out, float *__restrict__ lse)
{
    constexpr int NT = WAVES * 64;
    using Sm = FwdSmem<DQK, true, WAVES>;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int *redo_flag = Sm::redo_flags(smem);
    int *maps = redo_flag + kMaxItemsPerWg;

    // this workgroup's items: first + j + nx * t
    const int G = gridDim.x, xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int per = n_items >> 3, rem = n_items & 7;
    const int first = xcd * per + (xcd < rem ? xcd : rem), count = per + (xcd < rem ? 1 : 0);
    const int nx = (G >> 3) + ((G & 7) > xcd ? 1 : 0);
    const int my_n = j < count ? (count - j + nx - 1) / nx : 0;
    if (my_n == 0) return;
    const int item0 = item_base + first + j;

    if (!force_max) stream_items<DQK, ONES, WAVES>(g, nqblk, item0, nx, my_n, smem, q, k, v, fq, fk, out, lse);

    // Cold path: the noted items (every item under force_max) on the max-tracking general kernel body.
    __syncthreads();
    for (int t = 0; t < my_n; ++t) {
        if (!force_max && __builtin_amdgcn_readfirstlane(redo_flag[t]) == 0) continue;
        __syncthreads();
        const Item it = decode_item(g, item0 + nx * t, nqblk);
        const TokMap tok = fill_tok_map<NT>(g, it.w, maps);
        generic_item<DQK, WAVES, ONES, true>(g, it.u, it.blk, it.hd, tok, (bf16_t *)smem, 1, q, k, v, fq, fk, out, lse);
    }
}

// WAVES = 0: the general kernel (4 waves, 64-key tiles, one workgroup per item); 4 or 8: the
// streaming kernel (as many workgroups as the chip holds at once).
template <int DQK, bool ONES, int WAVES>
hipError_t launch(const Geo &g, int force_max, const void *q, const void *k, const void *v, const void *fq,
                  const void *fk, void *out, float *lse, hipStream_t st)
{
    constexpr bool FAST = WAVES != 0;
    constexpr int NW = FAST ? WAVES : 4;
    using Sm = FwdSmem<DQK, FAST, NW>;
    const int nqblk = (g.N + NW * 64 - 1) / (NW * 64);
    const int ntiles = (g.N + kTK - 1) / kTK;
    const int64_t items = g.units * nqblk;
    if constexpr (FAST) {
        const size_t dyn = Sm::TILE_BYTES + (size_t)NW * Sm::WAVE_ELEMS * sizeof(bf16_t) +
                           ((size_t)kMaxItemsPerWg + (size_t)3 * 2 * g.M) * sizeof(int);
        if (dyn > (size_t)kMaxDynLds) return hipErrorInvalidValue;
        auto kern = mfma_fwd_stream_kernel<DQK, ONES, NW>;
        int cus = 0;
        hipError_t e = prepare_kernel((const void *)kern, &cus);
        if (e != hipSuccess) return e;
        int per_cu = NW == 4 ? 2 : 1;               // what LDS and registers allow
        const int64_t slots = (int64_t)cus * per_cu;
        // (a launch hands a workgroup at most kMaxItemsPerWg items; larger problems take several launches)
        for (int64_t done = 0; done < items;) {
            const int64_t n = items - done < slots * kMaxItemsPerWg ? items - done : slots * kMaxItemsPerWg;
            const unsigned grid = (unsigned)(n < slots ? n : slots);
            hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), dyn, st, g, nqblk, (int)done, (int)n, force_max,
                               (const bf16_t *)q, (const bf16_t *)k, (const bf16_t *)v, (const bf16_t *)fq,
                               (const bf16_t *)fk, (bf16_t *)out, lse);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
            done += n;
        }
        return hipSuccess;
    } else {
        const size_t dyn = Sm::TILE_BYTES + (size_t)ntiles * kTK * sizeof(int);
        if (dyn > (size_t)kMaxDynLds) return hipErrorInvalidValue;
        auto kern = mfma_fwd_kernel<DQK, 4, ONES, false>;
        hipError_t e = prepare_kernel((const void *)kern, nullptr);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)items), dim3(NW * 64), dyn, st, g, nqblk, force_max, (const bf16_t *)q,
                           (const bf16_t *)k, (const bf16_t *)v, (const bf16_t *)fq, (const bf16_t *)fk, (bf16_t *)out,
                           lse);
        return hipGetLastError();
    }
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

// The streaming path needs whole tiles (128 keys with 4 waves, 256 with 8) and 32-bit byte
// offsets built with a 24-bit multiply.  Returns the number of waves per workgroup to run it
// with, 0 for the general kernel.  Eight waves (one workgroup per CU, each wave stages half as
// much per key block) are the faster form wherever the kernel variant fits its registers: head
// dims under 32 (the softmax denominator then comes out of the matrix cores) with 48 columns
// from 512 tokens per window on, with 64 columns from 4096 on (measured; config 5: 182 against
// 198 us).  The variants that sum the denominator on the vector ALU (d = 32) spill inside the
// loop with eight waves and stay at four.
static int fast_waves(const Geo &g)
{
    const int64_t tokens = (int64_t)g.B * g.H * g.W;
    const bool small_r = (g.d + g.r <= 48) ? (g.r <= 32) : true;
    if (!(g.r >= 4 && g.d >= 4 && g.N % 128 == 0 && g.N >= 256 && tokens < (1 << 24) && g.tstride * 2 < (1 << 24) &&
          tokens * g.tstride * 2 < ((int64_t)1 << 32) && small_r))
        return 0;
    if (g.N % 512 != 0) return 4;
    if (g.flags & RIB_FLAG_WIDE) return 8;
    const bool ones = g.d < 32, narrow = g.d + g.r <= 48;
    return ones && (narrow || g.N >= 4096) ? 8 : 4;
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
