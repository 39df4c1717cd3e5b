// RIB window attention for fp32 problems on the matrix cores (v_mfma_f32_32x32x2_f32).
//
// Same operator as include/rib_attn.h describes (paper Sec. 2.2; Sec. 3.1 Eq. 5-6), in fp32
// throughout: operands, products, accumulators and the softmax state are fp32, so the result
// meets the fp32 tolerance.  The vector-ALU kernels need one LDS operand per multiply-add
// and reach about a seventh of the fp32 peak; the fp32 MFMA has the same peak as the vector
// ALU but takes its operands once per 2048 multiply-adds.  It does occupy the vector ALU while
// it runs (measured: vector instructions between fp32 MFMAs add their full time, with one,
// two or three waves per SIMD), so a block costs its MFMA time plus its vector-instruction
// time, and everything around the MFMA chains is kept short.
//
// Layout of v_mfma_f32_32x32x2_f32 (D = A[32x2] * B[2x32] + C): lane l supplies
// A[l % 32][l / 32] and B[l / 32][l % 32] and holds D[8j + 4(l / 32) + i][l % 32] in register
// 4j + i.  Scores are computed TRANSPOSED (rows = streamed tokens, columns = this wave's 32
// stationary tokens), so every per-row quantity of the stationary side (running max, LSE,
// delta) is one value per lane, and an accumulator tile, read register by register, is
// already a B operand for the next product: the sum over the 32 streamed tokens runs over
// (register, lane half) pairs in whatever order, as long as the A operand is read in the
// same order.  No value ever moves between lanes except the row max / row sum halves.
//
// One workgroup = 4 waves = 128 consecutive window-local tokens of one (window, head) unit
// kept in registers; the other side is streamed through LDS in tiles of 64 tokens, fetched
// one tile ahead into registers, two LDS stages, one workgroup barrier per tile.  Any window of
// 32 or more tokens, any d <= 32, d + r <= 64.
#include "rib_common.h"

namespace rib {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kNT = 256;        // lanes per workgroup
constexpr int kRowsWg = 128;    // stationary tokens per workgroup (32 per wave)
constexpr int kTS = 64;         // streamed tokens per LDS tile
constexpr int kXS = 65;         // LDS row stride of the augmented tile (64 columns, odd stride)
constexpr int kYS = 33;         // LDS row stride of the value-side tile (32 columns)
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma(float a, float b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Eight A operands read ahead of the MFMA sequence that consumes them.
struct Pre {
    float v[8];
};

// acc += sum over i < CNT of A_i * B_i, where a_at(i) reads lane-wise A operands from LDS and
// b_at(i) names a register.  `pre` holds A_0..A_7 on entry; the operands of each further group of
// eight are read while the group before runs, and during the last group load_next(pre) reads the
// first eight operands of whatever sequence follows, so that a wave's matrix pipe never waits for
// LDS between sequences.  The scheduling barriers keep the compiler from hoisting every read of a
// 100-MFMA block to its top (which costs more registers than there are).
template <int CNT, class AF, class BF, class NF>
__device__ __forceinline__ void mfma_seq(f32x16 &acc, Pre &pre, AF a_at, BF b_at, NF load_next)
{
    constexpr int GS = 8, NG = CNT / GS;
    static_assert(CNT % GS == 0, "whole groups");
    float buf[2][GS];
#pragma unroll
    for (int i = 0; i < GS; ++i) buf[0][i] = pre.v[i];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        if (gi + 1 < NG) {
#pragma unroll
            for (int i = 0; i < GS; ++i) buf[(gi + 1) & 1][i] = a_at((gi + 1) * GS + i);
        } else {
            load_next(pre);
        }
#pragma unroll
        for (int i = 0; i < GS; ++i) acc = mfma(buf[gi & 1][i], b_at(gi * GS + i), acc);
        __builtin_amdgcn_sched_barrier(0);
    }
}
// register 4j + i of an accumulator tile <-> row 8j + 4*(lane half) + i: the row offset without the half
__device__ __forceinline__ constexpr int acc_row(int i) { return 8 * (i >> 2) + (i & 3); }

// Element t of the augmented vector of window-local token n (grid token tk): content
// channels scaled by sc, RIB features by sp, zero beyond d + r (Eq. 5).
__device__ __forceinline__ float aug_elem(const Geo &g, int hd, int n, int tk, const float *__restrict__ x,
                                          int64_t xstride, const float *__restrict__ f, float sc, float sp, int t)
{
    if (t < g.d) return x[(int64_t)tk * xstride + hd * g.d + t] * sc;
    if (t < g.d + g.r) return f[((int64_t)hd * g.N + n) * g.r + (t - g.d)] * sp;
    return 0.f;
}

// Registers that hold one streamed tile on its way from global memory to LDS.  Lane mapping of
// the grid tensors: lane (jj = tid / 32, c = tid % 32) fetches channel c of tokens jj, jj + 8, ...
// (whole token rows per wave pass); the RIB features of the tile's tokens are one contiguous
// run of 64 r floats, fetched linearly.
template <int DA>
struct TileRegs {
    static constexpr int FP = DA / 4;       // passes over the RIB run: 64 * r <= 64 * DA values, 256 per pass
    float xc[8], y[8], xf[FP], e0;
};

// The image a window lies in: base pointers of its tokens and the first token's index, so that
// offsets inside the image fit 32 bits (checked on the host).
struct ImgBase {
    const char *x, *y;      // streamed grid tensors, at the image's first token
    int tok0;               // b * H * W
};

// Request tile j0: content channels of x (token stride xs4 bytes), RIB features f and the value-side
// tensor y (stride ys4 bytes); for the key-side kernel also the tokens' LSE (times log2 e) and delta.
// Lanes beyond d and tokens beyond N fetch a clamped address (no divergent branches around the
// loads); tile_commit writes zeros for them.
template <int DA, bool EXTRA>
__device__ __forceinline__ void tile_request(TileRegs<DA> &rg, const Geo &g, int hd, int64_t u, int j0, const TokMap &tok,
                                             const ImgBase &ib, uint32_t xs4, uint32_t ys4, const float *__restrict__ f,
                                             const float *__restrict__ lse, const float *__restrict__ delta)
{
    const int tid = threadIdx.x, jj = tid >> 5, c = tid & 31;
    const int valid = g.N - j0 < kTS ? g.N - j0 : kTS;
    const uint32_t ch4 = (uint32_t)(hd * g.d + (c < g.d ? c : g.d - 1)) * 4u;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int n = jj + 8 * p;
        n = n < valid ? n : valid - 1;
        const uint32_t t = (uint32_t)(tok[j0 + n] - ib.tok0);
        rg.xc[p] = *(const float *)(ib.x + (t * xs4 + ch4));
        rg.y[p] = *(const float *)(ib.y + (t * ys4 + ch4));
    }
    const int cnt = valid * g.r;
    const float *fb = f + ((int64_t)hd * g.N + j0) * g.r;
#pragma unroll
    for (int p = 0; p < TileRegs<DA>::FP; ++p) {
        const int idx = p * kNT + tid;
        rg.xf[p] = idx < cnt ? fb[idx] : 0.f;
    }
    if (EXTRA) {
        const int n = tid & 63;
        rg.e0 = 0.f;
        if (tid < 64 && n < valid) rg.e0 = lse[u * g.N + j0 + n] * kLog2e;
        if (tid >= 64 && tid < 128 && n < valid) rg.e0 = delta[u * g.N + j0 + n];
    }
}

// Write the requested tile (it started at token j0) to LDS, content channels scaled by sc and RIB
// features by sp.  inv_r = ceil(2^32 / r) turns the position in the RIB run into (token, feature).
template <int DA, int XS, bool EXTRA>
__device__ __forceinline__ void tile_commit(const TileRegs<DA> &rg, const Geo &g, int j0, uint32_t inv_r, float sc, float sp,
                                            float *Xs, float *Ys, float *Es)
{
    const int tid = threadIdx.x, jj = tid >> 5, c = tid & 31;
    const int valid = g.N - j0 < kTS ? g.N - j0 : kTS;
    const bool cv = c < g.d;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        const bool ok = cv && jj + 8 * p < valid;
        if (cv) Xs[(jj + 8 * p) * XS + c] = ok ? rg.xc[p] * sc : 0.f;
        Ys[(jj + 8 * p) * kYS + c] = ok ? rg.y[p] : 0.f;
    }
    const int cnt = kTS * g.r;
#pragma unroll
    for (int p = 0; p < TileRegs<DA>::FP; ++p) {
        const int idx = p * kNT + tid;
        if (idx < cnt) {
            const int tkn = g.r == 1 ? idx : (int)__umulhi((uint32_t)idx, inv_r);     // 2^32 / 1 does not fit
            Xs[tkn * XS + g.d + (idx - tkn * g.r)] = rg.xf[p] * sp;
        }
    }
    if (EXTRA && tid < 128) Es[tid] = rg.e0;       // [0, 64) LSE * log2 e, [64, 128) delta
}

// blockIdx -> (unit, block of 128 stationary tokens), consecutive logical ids on one XCD so that
// the blocks of a unit share that XCD's L2.
__device__ __forceinline__ void unit_of_block(int nblk, int64_t &u, int &blk)
{
    const int G = gridDim.x, per = G >> 3, rem = G & 7, xcd = blockIdx.x & 7;
    const int logical = xcd * per + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    u = logical / nblk;
    blk = logical - (int)(u * nblk);
}

// Two stages of the streamed tile: while the waves work on one, the next is written to the other,
// one workgroup barrier per tile.  XS = row stride of the augmented tile (odd).
template <int XS>
struct Smem {
    float X[2][kTS * XS];
    float Y[2][kTS * kYS];
    float E[2][128];
    __attribute__((aligned(16))) int tokl[512];
};

// The staging code never writes columns d + r and up of the augmented tiles: they must read as zero.
template <int XS>
__device__ __forceinline__ void zero_x_tiles(float *Xs)
{
    for (int e = threadIdx.x; e < 2 * kTS * XS; e += kNT) Xs[e] = 0.f;
}

// Forward: Q_aug rows stationary (pre-multiplied by the scales and log2 e), K_aug / V streamed;
// online softmax with the running row max per lane.  Three workgroups per CU.
template <int DA>
__global__ __launch_bounds__(kNT, 3) void mfma_f32_fwd_kernel(Geo g, int nblk, uint32_t inv_r, const float *__restrict__ q,
                                                               const float *__restrict__ k, const float *__restrict__ v,
                                                               const float *__restrict__ fq, const float *__restrict__ fk,
                                                               float *__restrict__ out, float *__restrict__ lse)
{
    constexpr int XS = DA + 1;
    __shared__ Smem<XS> sm;
    int64_t u;
    int blk;
    unit_of_block(nblk, u, blk);
    const int w = (int)(u / g.heads), hd = (int)(u - (int64_t)w * g.heads);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;

    const TokMap tok = fill_tok_map<kNT>(g, w, sm.tokl);
    zero_x_tiles<XS>(sm.X[0]);
    __syncthreads();

    const int nt = (g.N + kTS - 1) / kTS;
    const int tok0 = (w / (g.nwx * g.nwy)) * g.H * g.W;
    const uint32_t ts4 = (uint32_t)g.tstride * 4u;
    const ImgBase ib = {(const char *)(k + (int64_t)tok0 * g.tstride), (const char *)(v + (int64_t)tok0 * g.tstride), tok0};
    TileRegs<DA> rg;
    tile_request<DA, false>(rg, g, hd, u, 0, tok, ib, ts4, ts4, fk, nullptr, nullptr);

    const int qi = blk * kRowsWg + wave * 32 + col;
    const bool live = qi < g.N;
    const int qc = live ? qi : g.N - 1;
    const int tq = tok[qc];
    float Qr[DA / 2];
#pragma unroll
    for (int t = 0; t < DA / 2; ++t)
        Qr[t] = aug_elem(g, hd, qc, tq, q, g.tstride, fq, g.scale_c * kLog2e, g.scale_p * kLog2e, 2 * t + hf);

    tile_commit<DA, XS, false>(rg, g, 0, inv_r, 1.f, 1.f, sm.X[0], sm.Y[0], sm.E[0]);
    if (nt > 1) tile_request<DA, false>(rg, g, hd, u, kTS, tok, ib, ts4, ts4, fk, nullptr, nullptr);
    __syncthreads();

    f32x16 O = {0};
    float m = -INFINITY, l = 0.f;
    for (int tile = 0; tile < nt; ++tile) {
        const int cur = tile & 1, j0 = tile * kTS;
        const float *Xc = sm.X[cur], *Yc = sm.Y[cur];
        Pre pre;
#pragma unroll
        for (int i = 0; i < 8; ++i) pre.v[i] = Xc[col * XS + hf + 2 * i];
#pragma unroll 1
        for (int kb = 0; kb < kTS / 32; ++kb) {
            const int key0 = j0 + kb * 32;
            if (key0 >= g.N) break;
            const float *Xb = Xc + (kb * 32 + col) * XS + hf;
            const float *Yb = Yc + (kb * 32 + 4 * hf) * kYS + col;
            f32x16 S = {0};
            mfma_seq<DA / 2>(S, pre, [&](int t) { return Xb[2 * t]; }, [&](int t) { return Qr[t]; },
                             [&](Pre &nx) {
#pragma unroll
                                 for (int i = 0; i < 8; ++i) nx.v[i] = Yb[acc_row(i) * kYS];
                             });
            if (key0 + 32 > g.N) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    if (key0 + acc_row(i) + 4 * hf >= g.N) S[i] = -INFINITY;
            }
            float mx = m;
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, S[i]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));     // finite: key0 < N is in this block or an earlier one
            const float alpha = __builtin_amdgcn_exp2f(m - mx);
            m = mx;
            float ps = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                S[i] = __builtin_amdgcn_exp2f(S[i] - mx);
                ps += S[i];
                O[i] *= alpha;
            }
            l = l * alpha + ps;
            mfma_seq<16>(O, pre, [&](int i) { return Yb[acc_row(i) * kYS]; }, [&](int i) { return S[i]; },
                         [&](Pre &nx) {
                             if (kb + 1 < kTS / 32) {
#pragma unroll
                                 for (int i = 0; i < 8; ++i) nx.v[i] = Xb[32 * XS + 2 * i];
                             }
                         });
        }
        if (tile + 1 < nt) {
            tile_commit<DA, XS, false>(rg, g, j0 + kTS, inv_r, 1.f, 1.f, sm.X[cur ^ 1], sm.Y[cur ^ 1], sm.E[cur ^ 1]);
            if (tile + 2 < nt)
                tile_request<DA, false>(rg, g, hd, u, j0 + 2 * kTS, tok, ib, ts4, ts4, fk, nullptr, nullptr);
        }
        __syncthreads();
    }
    l += __shfl_xor(l, 32);
    if (!live) return;
    const float inv = 1.f / l;
    const int64_t base = (int64_t)tq * g.C + hd * g.d;
    const float *gt = g.gate ? (const float *)g.gate + base : nullptr;
    float *raw = g.out_raw ? (float *)g.out_raw + base : nullptr;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = acc_row(i) + 4 * hf;
        if (c >= g.d) continue;
        const float o = O[i] * inv;
        if (gt) {       // CLA gate (Eq. 9) on the way out, the raw O beside it if asked for
            out[base + c] = o * gt[c];
            if (raw) raw[c] = o;
        } else {
            out[base + c] = o;
        }
    }
    if (lse != nullptr && hf == 0) lse[u * g.N + qi] = (m + log2f(l)) * kLn2;
}

// dQ and this unit's dF_q contribution: Q_aug, dO rows stationary, K_aug / V streamed.
//   S^T = K_aug Q_aug^T, dP^T = V dO^T, dS = P (dP - delta), dQ_aug^T += K_aug^T dS^T.
template <int DA>
__global__ __launch_bounds__(kNT, 2) void mfma_f32_dq_kernel(Geo g, int nblk, uint32_t inv_r, const float *__restrict__ q,
                                                              const float *__restrict__ k, const float *__restrict__ v,
                                                              const float *__restrict__ fq, const float *__restrict__ fk,
                                                              const float *__restrict__ dout, const float *__restrict__ lse,
                                                              const float *__restrict__ delta, float *__restrict__ dq,
                                                              float *__restrict__ dfq_part)
{
    constexpr int RB = DA > 32 ? 2 : 1;     // 32-row blocks of dQ_aug^T
    constexpr int XS = kXS;                 // all 64 columns: the second row block reads columns 32..63
    __shared__ Smem<XS> sm;
    int64_t u;
    int blk;
    unit_of_block(nblk, u, blk);
    const int w = (int)(u / g.heads), hd = (int)(u - (int64_t)w * g.heads);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;

    const TokMap tok = fill_tok_map<kNT>(g, w, sm.tokl);
    zero_x_tiles<XS>(sm.X[0]);      // zero operands beyond d + r, and finite (unused) rows of dQ_aug^T there
    __syncthreads();

    const int nt = (g.N + kTS - 1) / kTS;
    const int tok0 = (w / (g.nwx * g.nwy)) * g.H * g.W;
    const uint32_t ts4 = (uint32_t)g.tstride * 4u;
    const ImgBase ib = {(const char *)(k + (int64_t)tok0 * g.tstride), (const char *)(v + (int64_t)tok0 * g.tstride), tok0};
    TileRegs<DA> rg;
    tile_request<DA, false>(rg, g, hd, u, 0, tok, ib, ts4, ts4, fk, nullptr, nullptr);

    const int qi = blk * kRowsWg + wave * 32 + col;
    const bool live = qi < g.N;
    const int qc = live ? qi : g.N - 1;
    const int tq = tok[qc];
    float Qr[DA / 2], Gr[16];
#pragma unroll
    for (int t = 0; t < DA / 2; ++t)
        Qr[t] = aug_elem(g, hd, qc, tq, q, g.tstride, fq, g.scale_c * kLog2e, g.scale_p * kLog2e, 2 * t + hf);
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int c = 2 * t + hf;
        Gr[t] = c < g.d ? dout[(int64_t)tq * g.C + hd * g.d + c] : 0.f;
    }
    const float lse2 = lse[u * g.N + qc] * kLog2e, dl = delta[u * g.N + qc];

    tile_commit<DA, XS, false>(rg, g, 0, inv_r, 1.f, 1.f, sm.X[0], sm.Y[0], sm.E[0]);
    if (nt > 1) tile_request<DA, false>(rg, g, hd, u, kTS, tok, ib, ts4, ts4, fk, nullptr, nullptr);
    __syncthreads();

    f32x16 acc[RB];
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;

    for (int tile = 0; tile < nt; ++tile) {
        const int cur = tile & 1, j0 = tile * kTS;
        const float *Xc = sm.X[cur], *Yc = sm.Y[cur];
        Pre pre;
#pragma unroll
        for (int i = 0; i < 8; ++i) pre.v[i] = Xc[col * XS + hf + 2 * i];
#pragma unroll 1
        for (int kb = 0; kb < kTS / 32; ++kb) {
            if (j0 + kb * 32 >= g.N) break;
            // keys >= N are zero rows: their dS is finite and meets a zero K_aug row
            const float *Xb = Xc + (kb * 32 + col) * XS + hf;
            const float *Yb = Yc + (kb * 32 + col) * kYS + hf;
            const float *Xt = Xc + (kb * 32 + 4 * hf) * XS + col;
            f32x16 S = {0}, D = {0};
            mfma_seq<DA / 2>(S, pre, [&](int t) { return Xb[2 * t]; }, [&](int t) { return Qr[t]; },
                             [&](Pre &nx) {
#pragma unroll
                                 for (int i = 0; i < 8; ++i) nx.v[i] = Yb[2 * i];
                             });
            mfma_seq<16>(D, pre, [&](int t) { return Yb[2 * t]; }, [&](int t) { return Gr[t]; },
                         [&](Pre &nx) {
#pragma unroll
                             for (int i = 0; i < 8; ++i) nx.v[i] = Xt[acc_row(i) * XS];
                         });
#pragma unroll
            for (int i = 0; i < 16; ++i) S[i] = __builtin_amdgcn_exp2f(S[i] - lse2) * (D[i] - dl);
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                mfma_seq<16>(acc[b], pre, [&](int i) { return Xt[acc_row(i) * XS + 32 * b]; }, [&](int i) { return S[i]; },
                             [&](Pre &nx) {
                                 if (b + 1 < RB) {
#pragma unroll
                                     for (int i = 0; i < 8; ++i) nx.v[i] = Xt[acc_row(i) * XS + 32 * (b + 1)];
                                 } else if (kb + 1 < kTS / 32) {
#pragma unroll
                                     for (int i = 0; i < 8; ++i) nx.v[i] = Xb[32 * XS + 2 * i];
                                 }
                             });
            }
        }
        if (tile + 1 < nt) {
            tile_commit<DA, XS, false>(rg, g, j0 + kTS, inv_r, 1.f, 1.f, sm.X[cur ^ 1], sm.Y[cur ^ 1], sm.E[cur ^ 1]);
            if (tile + 2 < nt)
                tile_request<DA, false>(rg, g, hd, u, j0 + 2 * kTS, tok, ib, ts4, ts4, fk, nullptr, nullptr);
        }
        __syncthreads();
    }
    if (!live) return;
    float *dst = dq + (int64_t)tq * g.C + hd * g.d;
    float *fdst = dfq_part + (u * g.N + qi) * g.r;
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int c = 32 * b + acc_row(i) + 4 * hf;
            if (c < g.d) dst[c] = acc[b][i] * g.scale_c;
            else if (c < g.d + g.r) fdst[c - g.d] = acc[b][i] * g.scale_p;
        }
}

// dK, dV and this unit's dF_k contribution: K_aug, V rows stationary, Q_aug (scaled) / dO streamed
// together with the queries' LSE and delta.
//   S = Q_aug K_aug^T, dP = dO V^T, P = exp(S - LSE), dS = P (dP - delta),
//   dV^T += dO^T P, dK_aug^T += Q_aug^T dS.
template <int DA>
__global__ __launch_bounds__(kNT, 2) void mfma_f32_dkv_kernel(Geo g, int nblk, uint32_t inv_r, const float *__restrict__ q,
                                                               const float *__restrict__ k, const float *__restrict__ v,
                                                               const float *__restrict__ fq, const float *__restrict__ fk,
                                                               const float *__restrict__ dout, const float *__restrict__ lse,
                                                               const float *__restrict__ delta, float *__restrict__ dk,
                                                               float *__restrict__ dv, float *__restrict__ dfk_part)
{
    constexpr int RB = DA > 32 ? 2 : 1;
    constexpr int XS = kXS;
    __shared__ Smem<XS> sm;
    int64_t u;
    int blk;
    unit_of_block(nblk, u, blk);
    const int w = (int)(u / g.heads), hd = (int)(u - (int64_t)w * g.heads);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, hf = lane >> 5;

    const TokMap tok = fill_tok_map<kNT>(g, w, sm.tokl);
    zero_x_tiles<XS>(sm.X[0]);
    __syncthreads();

    const int nt = (g.N + kTS - 1) / kTS;
    const int tok0 = (w / (g.nwx * g.nwy)) * g.H * g.W;
    const uint32_t ts4 = (uint32_t)g.tstride * 4u;
    const ImgBase ib = {(const char *)(q + (int64_t)tok0 * g.tstride), (const char *)(dout + (int64_t)tok0 * g.C), tok0};
    TileRegs<DA> rg;
    tile_request<DA, true>(rg, g, hd, u, 0, tok, ib, ts4, (uint32_t)g.C * 4u, fq, lse, delta);

    const int ki = blk * kRowsWg + wave * 32 + col;
    const bool live = ki < g.N;
    const int kc = live ? ki : g.N - 1;
    const int tk = tok[kc];
    float Kr[DA / 2], Vr[16];
#pragma unroll
    for (int t = 0; t < DA / 2; ++t) Kr[t] = aug_elem(g, hd, kc, tk, k, g.tstride, fk, 1.f, 1.f, 2 * t + hf);
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        const int c = 2 * t + hf;
        Vr[t] = c < g.d ? v[(int64_t)tk * g.tstride + hd * g.d + c] : 0.f;
    }

    tile_commit<DA, XS, true>(rg, g, 0, inv_r, g.scale_c, g.scale_p, sm.X[0], sm.Y[0], sm.E[0]);
    if (nt > 1) tile_request<DA, true>(rg, g, hd, u, kTS, tok, ib, ts4, (uint32_t)g.C * 4u, fq, lse, delta);
    __syncthreads();

    f32x16 dKa[RB], dVa = {0};
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) dKa[b][i] = 0.f;

    for (int tile = 0; tile < nt; ++tile) {
        const int cur = tile & 1, i0 = tile * kTS;
        const float *Xc = sm.X[cur], *Yc = sm.Y[cur], *Ec = sm.E[cur];
        Pre pre;
#pragma unroll
        for (int i = 0; i < 8; ++i) pre.v[i] = Xc[col * XS + hf + 2 * i];
#pragma unroll 1
        for (int qb = 0; qb < kTS / 32; ++qb) {
            if (i0 + qb * 32 >= g.N) break;
            // queries >= N are zero rows with LSE = delta = 0: P = 1, dS = 0, and both meet zero rows
            const float *Xb = Xc + (qb * 32 + col) * XS + hf;
            const float *Yb = Yc + (qb * 32 + col) * kYS + hf;
            const float *Yt = Yc + (qb * 32 + 4 * hf) * kYS + col;
            const float *Xt = Xc + (qb * 32 + 4 * hf) * XS + col;
            f32x16 S = {0}, D = {0};
            mfma_seq<DA / 2>(S, pre, [&](int t) { return Xb[2 * t]; }, [&](int t) { return Kr[t]; },
                             [&](Pre &nx) {
#pragma unroll
                                 for (int i = 0; i < 8; ++i) nx.v[i] = Yb[2 * i];
                             });
            mfma_seq<16>(D, pre, [&](int t) { return Yb[2 * t]; }, [&](int t) { return Vr[t]; },
                         [&](Pre &nx) {
#pragma unroll
                             for (int i = 0; i < 8; ++i) nx.v[i] = Yt[acc_row(i) * kYS];
                         });
            // rows of S are queries: register 4j + i belongs to query 8j + 4hf + i of the block
            const float *Le = Ec + qb * 32 + 4 * hf, *De = Ec + 64 + qb * 32 + 4 * hf;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int rq = acc_row(i);
                const float p = __builtin_amdgcn_exp2f(fmaf(S[i], kLog2e, -Le[rq]));
                S[i] = p;
                D[i] = p * (D[i] - De[rq]);
            }
            mfma_seq<16>(dVa, pre, [&](int i) { return Yt[acc_row(i) * kYS]; }, [&](int i) { return S[i]; },
                         [&](Pre &nx) {
#pragma unroll
                             for (int i = 0; i < 8; ++i) nx.v[i] = Xt[acc_row(i) * XS];
                         });
#pragma unroll
            for (int b = 0; b < RB; ++b) {
                mfma_seq<16>(dKa[b], pre, [&](int i) { return Xt[acc_row(i) * XS + 32 * b]; }, [&](int i) { return D[i]; },
                             [&](Pre &nx) {
                                 if (b + 1 < RB) {
#pragma unroll
                                     for (int i = 0; i < 8; ++i) nx.v[i] = Xt[acc_row(i) * XS + 32 * (b + 1)];
                                 } else if (qb + 1 < kTS / 32) {
#pragma unroll
                                     for (int i = 0; i < 8; ++i) nx.v[i] = Xb[32 * XS + 2 * i];
                                 }
                             });
            }
        }
        if (tile + 1 < nt) {
            tile_commit<DA, XS, true>(rg, g, i0 + kTS, inv_r, g.scale_c, g.scale_p, sm.X[cur ^ 1], sm.Y[cur ^ 1], sm.E[cur ^ 1]);
            if (tile + 2 < nt)
                tile_request<DA, true>(rg, g, hd, u, i0 + 2 * kTS, tok, ib, ts4, (uint32_t)g.C * 4u, fq, lse, delta);
        }
        __syncthreads();
    }
    if (!live) return;
    float *kdst = dk + (int64_t)tk * g.C + hd * g.d;
    float *vdst = dv + (int64_t)tk * g.C + hd * g.d;
    float *fdst = dfk_part + (u * g.N + ki) * g.r;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int c = acc_row(i) + 4 * hf;
        if (c < g.d) vdst[c] = dVa[i];
    }
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int c = 32 * b + acc_row(i) + 4 * hf;
            if (c < g.d) kdst[c] = dKa[b][i];
            else if (c < g.d + g.r) fdst[c - g.d] = dKa[b][i];
        }
}

inline uint32_t inv_r_of(const Geo &g) { return g.r > 1 ? (uint32_t)((((uint64_t)1 << 32) + g.r - 1) / g.r) : 0u; }
inline int padded_da(const Geo &g) { return (g.d + g.r + 15) / 16 * 16; }

template <int DA>
hipError_t fwd_t(const Geo &g, const void *q, const void *k, const void *v, const void *fq, const void *fk, void *out,
                 float *lse, hipStream_t st)
{
    const int nblk = (g.N + kRowsWg - 1) / kRowsWg;
    hipLaunchKernelGGL((mfma_f32_fwd_kernel<DA>), dim3((unsigned)(g.units * nblk)), dim3(kNT), 0, st, g, nblk, inv_r_of(g),
                       (const float *)q, (const float *)k, (const float *)v, (const float *)fq, (const float *)fk,
                       (float *)out, lse);
    return hipGetLastError();
}

template <int DA>
hipError_t bwd_t(const Geo &g, const void *q, const void *k, const void *v, const void *fq, const void *fk,
                 const void *dout, const float *lse, const float *delta, void *dq, void *dk, void *dv, float *pq,
                 float *pk, hipStream_t st)
{
    const int nblk = (g.N + kRowsWg - 1) / kRowsWg;
    const dim3 grid((unsigned)(g.units * nblk));
    hipLaunchKernelGGL((mfma_f32_dkv_kernel<DA>), grid, dim3(kNT), 0, st, g, nblk, inv_r_of(g), (const float *)q, (const float *)k,
                       (const float *)v, (const float *)fq, (const float *)fk, (const float *)dout, lse, delta,
                       (float *)dk, (float *)dv, pk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((mfma_f32_dq_kernel<DA>), grid, dim3(kNT), 0, st, g, nblk, inv_r_of(g), (const float *)q, (const float *)k,
                       (const float *)v, (const float *)fq, (const float *)fk, (const float *)dout, lse, delta,
                       (float *)dq, pq);
    return hipGetLastError();
}

}  // namespace

// fp32 storage, head dim and augmented width within one / two 32-row blocks, and a window large
// enough to fill a 32-token block; everything else stays on the vector-ALU kernels.
bool mfma_f32_supported(const Geo &g, int dtype)
{
    const int64_t image_bytes = (int64_t)g.H * g.W * (g.tstride > g.C ? g.tstride : (int64_t)g.C) * 4;
    return dtype == RIB_F32 && !(g.flags & RIB_FLAG_VECTOR_ONLY) && g.d <= 32 && g.d + g.r <= 64 && g.N >= 32 &&
           g.M <= 256 && image_bytes < ((int64_t)1 << 32);
}

hipError_t launch_mfma_f32_fwd(const Geo &g, const void *q, const void *k, const void *v, const void *fq,
                               const void *fk, void *out, float *lse, hipStream_t st)
{
    switch (padded_da(g)) {
    case 16: return fwd_t<16>(g, q, k, v, fq, fk, out, lse, st);
    case 32: return fwd_t<32>(g, q, k, v, fq, fk, out, lse, st);
    case 48: return fwd_t<48>(g, q, k, v, fq, fk, out, lse, st);
    default: return fwd_t<64>(g, q, k, v, fq, fk, out, lse, st);
    }
}

hipError_t launch_mfma_f32_bwd(const Geo &g, const void *q, const void *k, const void *v, const void *fq,
                               const void *fk, const void *out, const void *dout, const float *lse, void *dq, void *dk,
                               void *dv, float *dfq, float *dfk, void *ws, hipStream_t st, void *gated_dout, void *dgate)
{
    const BwdWs l = bwd_ws_layout(g);
    float *delta = (float *)((char *)ws + l.delta_off);
    float *pq = (float *)((char *)ws + l.dfq_off);
    float *pk = (float *)((char *)ws + l.dfk_off);
    hipError_t e;
    if (g.gate) {
        e = launch_delta_gated(g, RIB_F32, out, dout, g.gate, delta, gated_dout, dgate, st);
        dout = gated_dout;
    } else {
        e = launch_delta(g, RIB_F32, out, dout, delta, st);
    }
    if (e != hipSuccess) return e;
    switch (padded_da(g)) {
    case 16: e = bwd_t<16>(g, q, k, v, fq, fk, dout, lse, delta, dq, dk, dv, pq, pk, st); break;
    case 32: e = bwd_t<32>(g, q, k, v, fq, fk, dout, lse, delta, dq, dk, dv, pq, pk, st); break;
    case 48: e = bwd_t<48>(g, q, k, v, fq, fk, dout, lse, delta, dq, dk, dv, pq, pk, st); break;
    default: e = bwd_t<64>(g, q, k, v, fq, fk, dout, lse, delta, dq, dk, dv, pq, pk, st); break;
    }
    if (e != hipSuccess) return e;
    return launch_reduce_df(g, pq, pk, dfq, dfk, st);
}

}  // namespace rib
