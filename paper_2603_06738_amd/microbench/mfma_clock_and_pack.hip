// Micro-benchmark behind three statements about gfx950 the forward kernel's design rests on:
//   1. the bf16 MFMA alone runs at its nominal rate with constant operands (13.5 ns per 32x32x16
//      instruction per SIMD) but at 17.7 ns with random operand bits: the chip lowers its clock
//      under the switching activity of the matrix pipe, so the sustained dense bf16 rate is about
//      three quarters of the nominal peak before anything else is considered;
//   2. what a 16-bit pack costs next to the MFMAs, for the candidate instructions (v_perm_b32,
//      v_pack_b32_f16 with op_sel, an SDWA move, v_cvt_pk_bf16_f32, ...);
//   3. the block mix (5 MFMA + 16 exp2 + 8 packs, software pipelined, registers only) with one or
//      two waves per SIMD: the ceiling of the forward loop's instruction mix.
// Registers only: no memory traffic inside the timed loops.
//
// build: hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//              -o mfma_clock_and_pack paper_2603_06738_amd/microbench/mfma_clock_and_pack.hip
// run:   ./mfma_clock_and_pack [waves per SIMD: 1 or 2, default 2]
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define MF(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b))
#define MF0(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=v"(acc) : "v"(a), "v"(b))
#define EXP(dst, src) asm volatile("v_exp_f32 %0, %1" : "=v"(dst) : "v"(src))

template <int OP>
__global__ __launch_bounds__(256) void rate(float* out, int iters)
{
    constexpr int NV = 32;
    float x[NV];
    for (int i = 0; i < NV; ++i) x[i] = threadIdx.x * 1e-4f + i * 0.01f + 1.0f;
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            float &a = x[i], &b = x[(i + 1) % NV];
            if (OP == 0) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(a) : "v"(a), "v"(b), "s"(0x07060302));
            if (OP == 1) asm volatile("v_pack_b32_f16 %0, %1, %2 op_sel:[1,1,0]" : "=v"(a) : "v"(b), "v"(a));
            if (OP == 2) asm volatile("v_mov_b32_sdwa %0, %1 dst_sel:WORD_0 dst_unused:UNUSED_PRESERVE src0_sel:WORD_1" : "+v"(a) : "v"(b));
            if (OP == 3) asm volatile("v_and_or_b32 %0, %1, %3, %2" : "=v"(a) : "v"(a), "v"(b), "s"(0xffff0000));
            if (OP == 4) asm volatile("v_bfi_b32 %0, %3, %1, %2" : "=v"(a) : "v"(a), "v"(b), "s"(0xffff0000));
            if (OP == 5) asm volatile("v_alignbit_b32 %0, %1, %2, 16" : "=v"(a) : "v"(a), "v"(b));
            if (OP == 6) asm volatile("v_lshrrev_b32 %0, 16, %1" : "=v"(a) : "v"(a));
            if (OP == 7) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(a) : "v"(a), "v"(b));
            if (OP == 8) asm volatile("v_exp_f32 %0, %1" : "=v"(a) : "v"(a));
            if (OP == 9) asm volatile("v_mul_f32 %0, %1, %1" : "=v"(a) : "v"(a));
            if (OP == 10) asm volatile("v_add_u32 %0, %1, %2" : "=v"(a) : "v"(a), "v"(b));
            if (OP == 11) asm volatile("v_exp_f16 %0, %1" : "=v"(a) : "v"(a));
            if (OP == 12) asm volatile("v_pk_mul_f16 %0, %1, %2" : "=v"(a) : "v"(a), "v"(b));
            if (OP == 13) asm volatile("v_cvt_pkrtz_f16_f32 %0, %1, %2" : "=v"(a) : "v"(a), "v"(b));
            if (OP == 14) asm volatile("v_max_f32 %0, %1, %2" : "=v"(a) : "v"(a), "v"(b));
            if (OP == 15) asm volatile("v_pk_add_u16 %0, %1, %2 op_sel:[1,0] op_sel_hi:[1,0]" : "=v"(a) : "v"(a), "v"(b));
        }
    }
    float s = __uint_as_float(acc);
    for (int i = 0; i < NV; ++i) s += x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// MFMA alone, NACC independent accumulators, constant or random operands
template <int NACC>
__global__ __launch_bounds__(256) void mfma_only(float* out, int iters, float scale)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        uint32_t h = (threadIdx.x * 2654435761u) ^ (i * 40503u + blockIdx.x * 9176u + 1u);
        h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
        float r1 = ((h & 0xffff) / 65536.0f - 0.5f) * scale, r2 = (((h >> 16) & 0xffff) / 65536.0f - 0.5f) * scale;
        a[i] = (__bf16)(scale == 0.f ? threadIdx.x * 0.001f + i : r1);
        b[i] = (__bf16)(scale == 0.f ? 0.01f * i : r2);
    }
    f32x16 c[NACC];
    for (int n = 0; n < NACC; ++n) for (int i = 0; i < 16; ++i) c[n][i] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 32; ++i) MF(c[i % NACC], a, b);
    }
    float s = 0;
    for (int n = 0; n < NACC; ++n) for (int i = 0; i < 16; ++i) s += c[n][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// exp only with random operands (does the clock drop without the matrix pipe?)
__global__ __launch_bounds__(256) void exp_only(float* out, int iters, float scale)
{
    float x[32], y[32];
    for (int i = 0; i < 32; ++i) {
        uint32_t h = (threadIdx.x * 2654435761u) ^ (i * 40503u + blockIdx.x * 9176u + 1u);
        h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
        x[i] = scale == 0.f ? 1.0f : ((h & 0xffff) / 65536.0f - 0.5f) * scale;
        y[i] = 0;
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 32; ++i) EXP(y[i], x[i]);
    }
    float s = 0;
    for (int i = 0; i < 32; ++i) s += y[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The block mix with a selectable pack: PK 0 = v_perm_b32, 1 = v_pack_b32_f16 op_sel, 2 = sdwa mov, 3 = none
template <int PK>
__device__ __forceinline__ uint32_t pack(float hi, float lo)
{
    uint32_t dst = 0;
    if (PK == 0) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(dst) : "v"(hi), "v"(lo), "s"(0x07060302));
    if (PK == 1) asm volatile("v_pack_b32_f16 %0, %1, %2 op_sel:[1,1,0]" : "=v"(dst) : "v"(lo), "v"(hi));
    if (PK == 2) { asm volatile("v_mov_b32_sdwa %0, %1 dst_sel:WORD_0 dst_unused:UNUSED_PRESERVE src0_sel:WORD_1" : "+v"(hi) : "v"(lo)); dst = __float_as_uint(hi); }
    if (PK == 3) dst = __float_as_uint(hi) ^ __float_as_uint(lo);
    return dst;
}
template <int PK>
__global__ __launch_bounds__(256) void block_mix(float* out, int iters, float scale)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        uint32_t h = (threadIdx.x * 2654435761u) ^ (i * 40503u + blockIdx.x * 9176u + 1u);
        h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
        float r1 = ((h & 0xffff) / 65536.0f - 0.5f) * scale, r2 = (((h >> 16) & 0xffff) / 65536.0f - 0.5f) * scale;
        a[i] = (__bf16)(scale == 0.f ? threadIdx.x * 0.001f + i : r1);
        b[i] = (__bf16)(scale == 0.f ? 0.01f * i : r2);
    }
    f32x16 S0, S1, O;
    for (int i = 0; i < 16; ++i) { S0[i] = 0; S1[i] = 0; O[i] = 0; }
    float e[16];
    u32x4 P0 = {0, 0, 0, 0}, P1 = {0, 0, 0, 0}, Q0 = {0, 0, 0, 0}, Q1 = {0, 0, 0, 0};
#define PERM(d, h, l) d = pack<PK>(h, l)
    for (int it = 0; it < iters; ++it) {
        MF0(S1, a, b); for (int i = 0; i < 4; ++i) EXP(e[i], S0[i]); PERM(P0[0], e[1], e[0]); PERM(P0[1], e[3], e[2]);
        MF(S1, a, b); for (int i = 4; i < 8; ++i) EXP(e[i], S0[i]); PERM(P0[2], e[5], e[4]); PERM(P0[3], e[7], e[6]);
        MF(S1, a, b); for (int i = 8; i < 12; ++i) EXP(e[i], S0[i]); PERM(P1[0], e[9], e[8]); PERM(P1[1], e[11], e[10]);
        MF(O, a, __builtin_bit_cast(bf16x8, Q0)); for (int i = 12; i < 16; ++i) EXP(e[i], S0[i]); PERM(P1[2], e[13], e[12]); PERM(P1[3], e[15], e[14]);
        MF(O, a, __builtin_bit_cast(bf16x8, Q1));
        MF0(S0, a, b); for (int i = 0; i < 4; ++i) EXP(e[i], S1[i]); PERM(Q0[0], e[1], e[0]); PERM(Q0[1], e[3], e[2]);
        MF(S0, a, b); for (int i = 4; i < 8; ++i) EXP(e[i], S1[i]); PERM(Q0[2], e[5], e[4]); PERM(Q0[3], e[7], e[6]);
        MF(S0, a, b); for (int i = 8; i < 12; ++i) EXP(e[i], S1[i]); PERM(Q1[0], e[9], e[8]); PERM(Q1[1], e[11], e[10]);
        MF(O, a, __builtin_bit_cast(bf16x8, P0)); for (int i = 12; i < 16; ++i) EXP(e[i], S1[i]); PERM(Q1[2], e[13], e[12]); PERM(Q1[3], e[15], e[14]);
        MF(O, a, __builtin_bit_cast(bf16x8, P1));
    }
    float s = 0;
    for (int i = 0; i < 16; ++i) s += S0[i] + S1[i] + O[i] + e[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s + __uint_as_float(P0[0] ^ P1[1] ^ Q0[2] ^ Q1[3]);
}

template <typename F>
static float best_ms(F f)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    f(); CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int r = 0; r < 3; ++r) {
        CK(hipEventRecord(e0)); f(); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    return best;
}

int main(int argc, char** argv)
{
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    float* out;
    CK(hipMalloc(&out, (size_t)cus * 8 * 256 * 4));
    const int wps = (argc > 1 ? atoi(argv[1]) : 2), blocks = cus * wps, iters = 20000;
    printf("%s, %d CUs, %d waves per SIMD, clock %d kHz\n", prop.gcnArchName, cus, wps, prop.clockRate);
    const char* names[] = {"v_perm_b32", "v_pack_b32_f16 op_sel", "v_mov_b32_sdwa", "v_and_or_b32", "v_bfi_b32", "v_alignbit_b32",
                           "v_lshrrev_b32", "v_cvt_pk_bf16_f32", "v_exp_f32", "v_mul_f32", "v_add_u32", "v_exp_f16", "v_pk_mul_f16",
                           "v_cvt_pkrtz_f16_f32", "v_max_f32", "v_pk_add_u16"};
    float t[16];
#define R(n) t[n] = best_ms([&] { rate<n><<<blocks, 256>>>(out, iters); }); printf("%-26s %.2f ns per wave instruction per SIMD\n", names[n], t[n] * 1e6 / ((double)iters * 32 * wps)); fflush(stdout);
    R(0) R(1) R(2) R(3) R(4) R(5) R(6) R(7) R(8) R(9) R(10) R(11) R(12) R(13) R(14) R(15)
    for (float scale : {0.f, 1.f}) {
        float m1 = best_ms([&] { mfma_only<1><<<blocks, 256>>>(out, iters, scale); });
        float m4 = best_ms([&] { mfma_only<4><<<blocks, 256>>>(out, iters, scale); });
        float ex = best_ms([&] { exp_only<<<blocks, 256>>>(out, iters, scale * 8.f); });
        printf("%s operands: MFMA alone %.2f ns (1 acc) %.2f ns (4 acc); v_exp_f32 alone %.2f ns\n", scale == 0.f ? "constant" : "random",
               m1 * 1e6 / ((double)iters * 32 * wps), m4 * 1e6 / ((double)iters * 32 * wps), ex * 1e6 / ((double)iters * 32 * wps));
        float b0 = best_ms([&] { block_mix<0><<<blocks, 256>>>(out, iters / 2, scale); });
        float b1 = best_ms([&] { block_mix<1><<<blocks, 256>>>(out, iters / 2, scale); });
        float b2 = best_ms([&] { block_mix<2><<<blocks, 256>>>(out, iters / 2, scale); });
        float b3 = best_ms([&] { block_mix<3><<<blocks, 256>>>(out, iters / 2, scale); });
        printf("  block mix ns per block per SIMD: perm %.1f  pack_f16 %.1f  sdwa %.1f  no pack (xor) %.1f\n",
               b0 * 1e6 / iters / wps, b1 * 1e6 / iters / wps, b2 * 1e6 / iters / wps, b3 * 1e6 / iters / wps);
        fflush(stdout);
    }
    // long run to see whether the clock settles lower: 10 back-to-back launches of the random mix
    for (int r = 0; r < 10; ++r) {
        float b0 = best_ms([&] { block_mix<0><<<blocks, 256>>>(out, iters / 2, 1.f); });
        printf("  run %d random perm mix %.1f ns\n", r, b0 * 1e6 / iters / wps);
    }
    return 0;
}
