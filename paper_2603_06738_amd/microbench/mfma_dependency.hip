// Micro-benchmark: does a chain of MFMAs that accumulate into ONE register block run slower than
// independent accumulators, with one and with two waves per SIMD, and how many v_exp_f32 ride along
// per MFMA for free?  Registers only.
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops -o mfma_dependency mfma_dependency.hip && ./mfma_dependency
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define MF(acc, a, b) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b))
// NACC independent accumulators used round-robin; VAL: number of independent v_exp per MFMA interleaved
template <int NACC, int VAL>
__global__ __launch_bounds__(256) void dep(float* out, int iters)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(threadIdx.x * 0.001f + i); b[i] = (__bf16)(0.01f * i); }
    f32x16 c[NACC];
    for (int n = 0; n < NACC; ++n) for (int i = 0; i < 16; ++i) c[n][i] = 0;
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = threadIdx.x * 1e-4f + i;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            MF(c[i % NACC], a, b);
#pragma unroll
            for (int v = 0; v < VAL; ++v) asm volatile("v_exp_f32 %0, %1" : "=v"(x[(i * VAL + v) % 8]) : "v"(x[(i * VAL + v) % 8]));
        }
    }
    float s = 0;
    for (int n = 0; n < NACC; ++n) for (int i = 0; i < 16; ++i) s += c[n][i];
    for (int i = 0; i < 8; ++i) s += x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
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
    for (int wps = 1; wps <= 2; ++wps) {
        const int blocks = cus * wps;
        const double n = (double)iters * 16 * wps;
        printf("waves/SIMD %d: ns per MFMA per SIMD\n", wps);
        printf("  chain of 1 acc          %.2f\n", best_ms([&] { dep<1, 0><<<blocks, 256>>>(out, iters); }) * 1e6 / n);
        printf("  2 accs                  %.2f\n", best_ms([&] { dep<2, 0><<<blocks, 256>>>(out, iters); }) * 1e6 / n);
        printf("  4 accs                  %.2f\n", best_ms([&] { dep<4, 0><<<blocks, 256>>>(out, iters); }) * 1e6 / n);
        printf("  1 acc + 3 exp per MFMA  %.2f\n", best_ms([&] { dep<1, 3><<<blocks, 256>>>(out, iters); }) * 1e6 / n);
        printf("  4 accs + 3 exp per MFMA %.2f\n", best_ms([&] { dep<4, 3><<<blocks, 256>>>(out, iters); }) * 1e6 / n);
        printf("  4 accs + 5 exp per MFMA %.2f\n", best_ms([&] { dep<4, 5><<<blocks, 256>>>(out, iters); }) * 1e6 / n);
    }
    CK(hipDeviceSynchronize());
    return 0;
}
