// Micro-benchmark behind the ceiling quoted for the forward kernel: how fast can one
// gfx950 SIMD issue the instruction mix of one 32x32 attention block
//   5 x v_mfma_f32_32x32x16_bf16  +  16 x v_exp_f32  +  8 x v_perm_b32
// with 2 waves per SIMD, for constant operands and for random operands (switching
// activity lowers the clock), plus single-instruction issue rates.  Registers only: no
// memory traffic inside the timed loops.
//
// build: hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//              -o issue_mix paper_2603_06738_amd/microbench/issue_mix.hip
// run:   ./issue_mix
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
#define PERM(dst, hi, lo) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(dst) : "v"(hi), "v"(lo), "s"(0x07060302))

// One attention block per half iteration, software pipelined as in the kernel: the exp2
// of block s read the scores produced one step earlier, the PV MFMAs read the packed
// probabilities of the step before.
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

// OP: 0 v_exp_f32, 1 v_perm_b32, 2 v_cvt_pk_bf16_f32, 3 v_mul_f32, 4 v_fma_f32, 5 v_max3_f32, 6 MFMA 32x32x16 bf16
template <int OP>
__global__ __launch_bounds__(256) void rate(float* out, int iters)
{
    constexpr int NV = 32;
    float x[NV];
    for (int i = 0; i < NV; ++i) x[i] = threadIdx.x * 1e-4f + i * 0.01f;
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f + i); b[i] = (__bf16)(0.01f * i); }
    f32x16 c[4];
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) c[n][i] = 0;
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            if (OP == 0) asm volatile("v_exp_f32 %0, %1" : "=v"(x[i]) : "v"(x[i]));
            if (OP == 1) asm volatile("v_perm_b32 %0, %1, %2, %1" : "=v"(x[i]) : "v"(x[i]), "v"(x[(i + 1) % NV]));
            if (OP == 2) { uint32_t r; asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(x[i]), "v"(x[(i + 1) % NV])); acc ^= r; }
            if (OP == 3) asm volatile("v_mul_f32 %0, %1, %1" : "=v"(x[i]) : "v"(x[i]));
            if (OP == 4) asm volatile("v_fma_f32 %0, %1, %1, %1" : "=v"(x[i]) : "v"(x[i]));
            if (OP == 5) asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(x[i]) : "v"(x[i]), "v"(x[(i + 1) % NV]), "v"(x[(i + 2) % NV]));
            if (OP == 6) MF(c[i % 4], a, b);
        }
    }
    float s = __uint_as_float(acc);
    for (int i = 0; i < NV; ++i) s += x[i];
    for (int n = 0; n < 4; ++n) for (int i = 0; i < 16; ++i) s += c[n][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
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

int main()
{
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    float* out;
    CK(hipMalloc(&out, (size_t)cus * 8 * 256 * 4));
    const int wps = 2, blocks = cus * wps, iters = 20000;
    printf("%s, %d CUs, %d waves per SIMD\n", prop.gcnArchName, cus, wps);
    const char* names[] = {"v_exp_f32", "v_perm_b32", "v_cvt_pk_bf16_f32", "v_mul_f32", "v_fma_f32", "v_max3_f32", "v_mfma_f32_32x32x16_bf16"};
    float t[7];
    t[0] = best_ms([&] { rate<0><<<blocks, 256>>>(out, iters); });
    t[1] = best_ms([&] { rate<1><<<blocks, 256>>>(out, iters); });
    t[2] = best_ms([&] { rate<2><<<blocks, 256>>>(out, iters); });
    t[3] = best_ms([&] { rate<3><<<blocks, 256>>>(out, iters); });
    t[4] = best_ms([&] { rate<4><<<blocks, 256>>>(out, iters); });
    t[5] = best_ms([&] { rate<5><<<blocks, 256>>>(out, iters); });
    t[6] = best_ms([&] { rate<6><<<blocks, 256>>>(out, iters); });
    for (int i = 0; i < 7; ++i)
        printf("%-26s %.2f ns per wave instruction per SIMD\n", names[i], t[i] * 1e6 / ((double)iters * 32 * wps));
    for (float scale : {0.f, 1.f}) {
        float ms = best_ms([&] { block_mix<<<blocks, 256>>>(out, iters / 2, scale); });
        double ns = ms * 1e6 / iters / wps;
        printf("block mix (5 MFMA + 16 exp2 + 8 perm), %s operands: %.1f ns per 32x32 block per SIMD"
               " => %.0f TFLOP/s of unpadded attention flop on %d SIMDs\n",
               scale == 0.f ? "constant" : "random", ns, 155648.0 * cus * 4 / ns * 1e-3, cus * 4);
    }
    return 0;
}
