// Does it matter HOW the two waves of a SIMD interleave the forward loop's instruction mix (5 MFMA + 16 exp2 +
// 8 packs per 32x32 block), and does a workgroup barrier every 16 blocks cost anything by re-aligning them?
// Registers only, 8-wave workgroups, one per CU.  Variants: the fine interleave the kernel uses (MFMA; 4 exp2;
// 2 packs), coarse phases (5 MFMAs, then 16 exp2 + 8 packs), raised priority in the MFMA phase, the second wave of
// a SIMD started half a block ahead, a short sleep of the second wave after each barrier.
// Result on gfx950: no variant differs by more than a few per cent (94-106 ns per block per SIMD with constant
// operands, 120-125 ns with random ones), barrier or not: the mix itself is arbitration-proof.  What the real
// kernel loses against this figure comes from what the mix leaves out (operand reads, staging, item boundaries).
//
// build: hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//              -o wave_pair_phases paper_2603_06738_amd/microbench/wave_pair_phases.hip
// run:   ./wave_pair_phases
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
#define PERM(d, h, l) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(d) : "v"(h), "v"(l), "s"(0x07060302))
#define PRIO(n) asm volatile("s_setprio " #n)
#define SLEEP1 asm volatile("s_sleep 1")

// MODE 0: fine interleave (MFMA; 4 exp; 2 perm) as the forward kernel has it
// MODE 1: coarse phases: 5 MFMAs, then 16 exp + 8 perm
// MODE 2: coarse phases with s_setprio 1 during the MFMA phase
// MODE 3: coarse, waves 4..7 start with the vector phase (anti-phase by construction), no priorities
// MODE 4: as 3 with s_setprio 1 during the MFMA phase
// MODE 5: fine interleave, waves 4..7 sleep 64 clk after each barrier
template <int MODE, int BPB, bool BAR>
__global__ __launch_bounds__(512) void mix(float* out, int iters, float scale)
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
    for (int i = 0; i < 16; ++i) e[i] = 0;
    u32x4 P0 = {0, 0, 0, 0}, P1 = {0, 0, 0, 0}, Q0 = {0, 0, 0, 0}, Q1 = {0, 0, 0, 0};
    const bool hi = __builtin_amdgcn_readfirstlane(threadIdx.x >> 8) != 0;
#define VGRP(S, i0, D, j0) { for (int i = i0; i < i0 + 4; ++i) EXP(e[i], S[i]); PERM(D[j0], e[i0 + 1], e[i0]); PERM(D[j0 + 1], e[i0 + 3], e[i0 + 2]); }
#define VPHASE(S, DA, DB) { VGRP(S, 0, DA, 0) VGRP(S, 4, DA, 2) VGRP(S, 8, DB, 0) VGRP(S, 12, DB, 2) }
#define MPHASE(SN, PA, PB) { MF0(SN, a, b); MF(SN, a, b); MF(SN, a, b); MF(O, a, __builtin_bit_cast(bf16x8, PA)); MF(O, a, __builtin_bit_cast(bf16x8, PB)); }
    if ((MODE == 3 || MODE == 4) && hi) { VPHASE(S0, P0, P1) }      // half a block ahead
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int blk = 0; blk < BPB; blk += 2) {
            if (MODE == 0 || MODE == 5) {
                MF0(S1, a, b); VGRP(S0, 0, P0, 0)
                MF(S1, a, b); VGRP(S0, 4, P0, 2)
                MF(S1, a, b); VGRP(S0, 8, P1, 0)
                MF(O, a, __builtin_bit_cast(bf16x8, Q0)); VGRP(S0, 12, P1, 2)
                MF(O, a, __builtin_bit_cast(bf16x8, Q1));
                MF0(S0, a, b); VGRP(S1, 0, Q0, 0)
                MF(S0, a, b); VGRP(S1, 4, Q0, 2)
                MF(S0, a, b); VGRP(S1, 8, Q1, 0)
                MF(O, a, __builtin_bit_cast(bf16x8, P0)); VGRP(S1, 12, Q1, 2)
                MF(O, a, __builtin_bit_cast(bf16x8, P1));
            } else {
                if (MODE == 2 || MODE == 4) PRIO(1);
                MPHASE(S1, Q0, Q1)
                if (MODE == 2 || MODE == 4) PRIO(0);
                VPHASE(S0, P0, P1)
                if (MODE == 2 || MODE == 4) PRIO(1);
                MPHASE(S0, P0, P1)
                if (MODE == 2 || MODE == 4) PRIO(0);
                VPHASE(S1, Q0, Q1)
            }
        }
        if (BAR) {
            __syncthreads();
            if (MODE == 5 && hi) SLEEP1;
        }
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

int main()
{
    hipDeviceProp_t prop;
    CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    float* out;
    CK(hipMalloc(&out, (size_t)cus * 512 * 4));
    constexpr int BPB = 16;
    const int iters = 1500;      // x 16 blocks per wave
    for (float scale : {0.f, 1.f}) {
        printf("%s operands; ns per block per SIMD (2 waves per SIMD, 8-wave workgroups)\n", scale == 0.f ? "constant" : "random");
#define RUN(M, B, label) { float t = best_ms([&] { mix<M, BPB, B><<<cus, 512>>>(out, iters, scale); }); printf("  %-58s %s: %.1f\n", label, B ? "barrier every 16 blocks" : "no barrier", t * 1e6 / ((double)iters * BPB * 2)); fflush(stdout); }
        RUN(0, false, "fine interleave") RUN(0, true, "fine interleave")
        RUN(5, true, "fine interleave, waves 4-7 sleep 64 clk after the barrier")
        RUN(1, false, "coarse phases") RUN(1, true, "coarse phases")
        RUN(2, false, "coarse phases, prio 1 in the MFMA phase") RUN(2, true, "coarse phases, prio 1 in the MFMA phase")
        RUN(3, false, "coarse, waves 4-7 half a block ahead") RUN(3, true, "coarse, waves 4-7 half a block ahead")
        RUN(4, false, "coarse, half a block ahead, prio 1 in MFMA phase") RUN(4, true, "coarse, half a block ahead, prio 1 in MFMA phase")
    }
    return 0;
}
