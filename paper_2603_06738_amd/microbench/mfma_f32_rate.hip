// Micro-benchmark: sustained rate of v_mfma_f32_32x32x2_f32 (the fp32 matrix instruction the fp32
// kernels are built on), registers only, with constant and with random operands, one to three
// waves per SIMD, accumulating into one register block or into two alternately; and whether
// independent vector instructions (v_fma_f32, v_exp_f32) issued between the MFMAs ride along for
// free, as they do beside the bf16 MFMAs, or add their own time.
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops -o mfma_f32_rate mfma_f32_rate.hip && ./mfma_f32_rate
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define MF(acc, a, b) asm volatile("v_mfma_f32_32x32x2_f32 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b))
template <int NACC, bool RANDOM>
__global__ __launch_bounds__(256) void rate(float* out, int iters)
{
    float a[8], b[8];
    uint32_t s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int i = 0; i < 8; ++i) {
        s = s * 1664525u + 1013904223u;
        a[i] = RANDOM ? (float)(int)(s >> 8) * (1.f / 8388608.f) - 1.f : 1.f;
        s = s * 1664525u + 1013904223u;
        b[i] = RANDOM ? (float)(int)(s >> 8) * (1.f / 8388608.f) - 1.f : 0.5f;
    }
    f32x16 c[NACC];
    for (int n = 0; n < NACC; ++n) for (int i = 0; i < 16; ++i) c[n][i] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) MF(c[i % NACC], a[i & 7], b[(i * 3) & 7]);
    }
    float t = 0;
    for (int n = 0; n < NACC; ++n) for (int i = 0; i < 16; ++i) t += c[n][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = t;
}
// VAL independent vector instructions after every MFMA (EXP: v_exp_f32, else v_fma_f32)
template <int VAL, bool EXP>
__global__ __launch_bounds__(256) void mix(float* out, int iters)
{
    float a = threadIdx.x * 0.001f, b = 0.5f, x[8];
    for (int i = 0; i < 8; ++i) x[i] = threadIdx.x * 1e-4f + i;
    f32x16 c;
    for (int i = 0; i < 16; ++i) c[i] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            MF(c, a, b);
#pragma unroll
            for (int v = 0; v < VAL; ++v) {
                if (EXP) asm volatile("v_exp_f32 %0, %1" : "=v"(x[(i * VAL + v) % 8]) : "v"(x[(i * VAL + v) % 8]));
                else asm volatile("v_fma_f32 %0, %1, %1, %0" : "+v"(x[(i * VAL + v) % 8]) : "v"(b));
            }
        }
    }
    float t = 0;
    for (int i = 0; i < 16; ++i) t += c[i];
    for (int i = 0; i < 8; ++i) t += x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = t;
}
template <typename F> static float best_ms(F f)
{
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    f(); hipDeviceSynchronize();
    float best = 1e30f;
    for (int r = 0; r < 3; ++r) { hipEventRecord(e0); f(); hipEventRecord(e1); hipEventSynchronize(e1); float ms; hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms; }
    return best;
}
int main()
{
    hipDeviceProp_t prop; CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    float* out; CK(hipMalloc(&out, (size_t)cus * 8 * 256 * 4));
    const int iters = 4000;
    for (int wps = 1; wps <= 3; ++wps) {
        const int blocks = cus * wps;
        const double n = (double)iters * 16 * wps;                        // MFMAs per SIMD
        const double flop = n * 4096.0 * cus * 4;                          // 32*32*2*2 per MFMA
        auto line = [&](const char* what, float ms) {
            printf("  %-34s %6.2f ns per MFMA per SIMD  %6.1f TFLOP/s\n", what, ms * 1e6 / n, flop / (ms * 1e-3) / 1e12);
        };
        printf("waves/SIMD %d\n", wps);
        line("1 accumulator, constant operands", best_ms([&] { rate<1, false><<<blocks, 256>>>(out, iters); }));
        line("2 accumulators, constant operands", best_ms([&] { rate<2, false><<<blocks, 256>>>(out, iters); }));
        line("1 accumulator, random operands", best_ms([&] { rate<1, true><<<blocks, 256>>>(out, iters); }));
        line("2 accumulators, random operands", best_ms([&] { rate<2, true><<<blocks, 256>>>(out, iters); }));
        line("+ 4 v_fma_f32 per MFMA", best_ms([&] { mix<4, false><<<blocks, 256>>>(out, iters); }));
        line("+ 8 v_fma_f32 per MFMA", best_ms([&] { mix<8, false><<<blocks, 256>>>(out, iters); }));
        line("+ 2 v_exp_f32 per MFMA", best_ms([&] { mix<2, true><<<blocks, 256>>>(out, iters); }));
        line("+ 4 v_exp_f32 per MFMA", best_ms([&] { mix<4, true><<<blocks, 256>>>(out, iters); }));
    }
    CK(hipDeviceSynchronize());
    return 0;
}
