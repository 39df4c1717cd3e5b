// Micro-benchmark: register-only model of one 32 x 32 block of the dQ backward kernel (3 + 2 score
// MFMAs -> 16 exp2, 16 multiplies, 8 packs on their results -> 4 gradient MFMAs on the packs), as a
// dependent chain and software-pipelined, with one and with two waves per SIMD.
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops -o bwd_block_model bwd_block_model.hip && ./bwd_block_model
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
__device__ __forceinline__ uint32_t tp(float lo, float hi) { return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u); }
__device__ __forceinline__ bf16x8 asb(uint32_t a, uint32_t b, uint32_t c, uint32_t d) { uint4 w = {a, b, c, d}; return __builtin_bit_cast(bf16x8, w); }
// One dq-like block per iteration, registers only: S = 3 MFMA, D = 2 MFMA, 16 exp2 * D, 8 packs, 4 gradient MFMAs.
// MODE 0: all; 1: MFMAs only (packs replaced by bit casts of S, D); 2: vector work only (no MFMA: S, D from registers)
template <int MODE>
__global__ __launch_bounds__(256, 2) void blockchain(float *out, int iters)
{
    bf16x8 a[3], q[3], av[2], gb[2], at[2][2];
    for (int t = 0; t < 3; ++t) for (int i = 0; i < 8; ++i) { a[t][i] = (__bf16)(0.01f * (threadIdx.x % 7 + i + t)); q[t][i] = (__bf16)(0.02f * (i - t)); }
    for (int t = 0; t < 2; ++t) for (int i = 0; i < 8; ++i) { av[t][i] = (__bf16)(0.03f * i); gb[t][i] = (__bf16)(0.01f * (t + 1)); at[0][t][i] = (__bf16)(0.05f * i); at[1][t][i] = (__bf16)(0.04f * i); }
    f32x16 acc[2] = {{0}, {0}};
    const f32x16 zero = {0};
    f32x16 S = zero, D = zero;
    for (int it = 0; it < iters; ++it) {
        if (MODE != 2) {
            S = mfma(a[0], q[0], zero); S = mfma(a[1], q[1], S); S = mfma(a[2], q[2], S);
            D = mfma(av[0], gb[0], zero); D = mfma(av[1], gb[1], D);
        } else {
            for (int i = 0; i < 16; ++i) { S[i] = acc[0][i] * 0.5f; D[i] = acc[1][i] * 0.25f; }
        }
        uint32_t w[8];
        for (int i = 0; i < 16; i += 2) {
            if (MODE == 1) w[i >> 1] = __float_as_uint(S[i]) ^ __float_as_uint(D[i + 1]);
            else w[i >> 1] = tp(__builtin_amdgcn_exp2f(S[i]) * D[i], __builtin_amdgcn_exp2f(S[i + 1]) * D[i + 1]);
        }
        if (MODE != 2) {
            const bf16x8 B0 = asb(w[0], w[1], w[2], w[3]), B1 = asb(w[4], w[5], w[6], w[7]);
            for (int mb = 0; mb < 2; ++mb) { acc[mb] = mfma(at[mb][0], B0, acc[mb]); acc[mb] = mfma(at[mb][1], B1, acc[mb]); }
        } else {
            for (int i = 0; i < 8; ++i) { acc[0][i] += __uint_as_float(w[i]); acc[1][i] += __uint_as_float(w[i] << 16); }
        }
        // make a's depend on nothing; perturb q so the compiler cannot hoist the score MFMAs
        q[0] = asb(w[0] & 0x3f003f00u, w[1] & 0x3f003f00u, 0x3c003c00u, 0x3c003c00u);
    }
    float s = 0;
    for (int i = 0; i < 16; ++i) s += acc[0][i] + acc[1][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
// software-pipelined form: scores of block b+1, vector work of block b, gradient MFMAs of block b-1
__global__ __launch_bounds__(256, 2) void pipelined(float *out, int iters)
{
    bf16x8 a[3], q[3], av[2], gb[2], at[2][2];
    for (int t = 0; t < 3; ++t) for (int i = 0; i < 8; ++i) { a[t][i] = (__bf16)(0.01f * (threadIdx.x % 7 + i + t)); q[t][i] = (__bf16)(0.02f * (i - t)); }
    for (int t = 0; t < 2; ++t) for (int i = 0; i < 8; ++i) { av[t][i] = (__bf16)(0.03f * i); gb[t][i] = (__bf16)(0.01f * (t + 1)); at[0][t][i] = (__bf16)(0.05f * i); at[1][t][i] = (__bf16)(0.04f * i); }
    f32x16 acc[2] = {{0}, {0}};
    const f32x16 zero = {0};
    f32x16 S[2], D[2];
    uint32_t w[2][8];
    for (int i = 0; i < 8; ++i) w[1][i] = 0x3c003c00u;
    S[0] = mfma(a[0], q[0], zero); S[0] = mfma(a[1], q[1], S[0]); S[0] = mfma(a[2], q[2], S[0]);
    D[0] = mfma(av[0], gb[0], zero); D[0] = mfma(av[1], gb[1], D[0]);
    for (int it = 0; it < iters; it += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int cs = h, ns = h ^ 1;
            // scores of the next block (operands perturbed with the packs of two blocks ago so nothing hoists)
            q[0] = asb(w[ns][0] & 0x3f003f00u, w[ns][1] & 0x3f003f00u, 0x3c003c00u, 0x3c003c00u);
            S[ns] = mfma(a[0], q[0], zero); S[ns] = mfma(a[1], q[1], S[ns]); S[ns] = mfma(a[2], q[2], S[ns]);
            D[ns] = mfma(av[0], gb[0], zero); D[ns] = mfma(av[1], gb[1], D[ns]);
            // gradient MFMAs of the previous block
            const bf16x8 B0 = asb(w[ns][0], w[ns][1], w[ns][2], w[ns][3]), B1 = asb(w[ns][4], w[ns][5], w[ns][6], w[ns][7]);
            for (int mb = 0; mb < 2; ++mb) { acc[mb] = mfma(at[mb][0], B0, acc[mb]); acc[mb] = mfma(at[mb][1], B1, acc[mb]); }
            // vector work of this block
            for (int i = 0; i < 16; i += 2)
                w[cs][i >> 1] = tp(__builtin_amdgcn_exp2f(S[cs][i]) * D[cs][i], __builtin_amdgcn_exp2f(S[cs][i + 1]) * D[cs][i + 1]);
            // interleave: one MFMA, two exp2, three other vector instructions
            for (int k = 0; k < 9; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
            }
        }
    }
    float s = 0;
    for (int i = 0; i < 16; ++i) s += acc[0][i] + acc[1][i] + S[0][i] + D[0][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
template <typename F> static float best_ms(F f)
{
    hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    f(); (void)hipDeviceSynchronize();
    float best = 1e30f;
    for (int r = 0; r < 3; ++r) { (void)hipEventRecord(e0); f(); (void)hipEventRecord(e1); (void)hipEventSynchronize(e1); float ms; (void)hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms; }
    return best;
}
int main()
{
    float *out; if (hipMalloc(&out, 1 << 24) != hipSuccess) return 1;
    const int iters = 20000;
    for (int wps = 1; wps <= 2; ++wps) {
        const int blocks = 256 * wps;
        const double n = (double)iters * wps;
        printf("waves/SIMD %d, ns per dq-like block per SIMD: all %.1f, MFMA only %.1f, vector only %.1f\n", wps,
               best_ms([&] { blockchain<0><<<blocks, 256>>>(out, iters); }) * 1e6 / n,
               best_ms([&] { blockchain<1><<<blocks, 256>>>(out, iters); }) * 1e6 / n,
               best_ms([&] { blockchain<2><<<blocks, 256>>>(out, iters); }) * 1e6 / n);
        printf("   software-pipelined: %.1f\n", best_ms([&] { pipelined<<<blocks, 256>>>(out, iters); }) * 1e6 / n);
    }
    return hipDeviceSynchronize() == hipSuccess ? 0 : 1;
}
