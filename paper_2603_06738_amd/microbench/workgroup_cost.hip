// Micro-benchmark: what one round of workgroups costs beyond the work inside them, for a kernel with
// the footprint of the attention kernels (256 threads, 70 KB of LDS, two workgroups per CU): a timed
// spin per workgroup, 1 / 6.75 / 27 rounds.
//   hipcc --offload-arch=gfx950 -O3 -o workgroup_cost workgroup_cost.hip && ./workgroup_cost
#include <hip/hip_runtime.h>
#include <cstdio>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
// empty-ish kernel with the register and LDS footprint of the forward fast kernel
template <int SPIN>
__global__ __launch_bounds__(256, 2) void k(float *out, int n)
{
    extern __shared__ float lds[];
    float acc[200];
#pragma unroll
    for (int i = 0; i < 200; ++i) acc[i] = threadIdx.x + i;
    lds[threadIdx.x] = acc[5];
    __syncthreads();
    if (SPIN) {
        const unsigned long long t0 = wall_clock64();
        while (wall_clock64() - t0 < (unsigned long long)SPIN) __builtin_amdgcn_s_sleep(8);
    }
    float s = lds[(threadIdx.x + 1) & 255];
    if (n == 12345) {
#pragma unroll
        for (int i = 0; i < 200; ++i) s += acc[i] * out[i];
        out[blockIdx.x * 256 + threadIdx.x] = s;
    }
}
template <typename F> static float best_ms(F f)
{
    hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    f(); (void)hipDeviceSynchronize();
    float best = 1e30f;
    for (int r = 0; r < 5; ++r) { (void)hipEventRecord(e0); f(); (void)hipEventRecord(e1); (void)hipEventSynchronize(e1); float ms; (void)hipEventElapsedTime(&ms, e0, e1); if (ms < best) best = ms; }
    return best;
}
int main()
{
    float *out; CK(hipMalloc(&out, 1 << 24));
    const size_t lds = 70 * 1024;
    CK(hipFuncSetAttribute((const void *)k<0>, hipFuncAttributeMaxDynamicSharedMemorySize, 158 * 1024));
    CK(hipFuncSetAttribute((const void *)k<1000>, hipFuncAttributeMaxDynamicSharedMemorySize, 158 * 1024));
    CK(hipFuncSetAttribute((const void *)k<2000>, hipFuncAttributeMaxDynamicSharedMemorySize, 158 * 1024));
    for (int wgs : {512, 3456, 13824}) {
        float t0 = best_ms([&] { k<0><<<wgs, 256, lds>>>(out, 0); });
        float t1 = best_ms([&] { k<1000><<<wgs, 256, lds>>>(out, 0); });   // 10 us of spinning per workgroup (100 MHz clock)
        float t2 = best_ms([&] { k<2000><<<wgs, 256, lds>>>(out, 0); });
        printf("%5d workgroups (%.2f rounds of 512): empty %.1f us, 10us-spin %.1f us, 20us-spin %.1f us\n", wgs, wgs / 512.0, t0 * 1e3, t1 * 1e3, t2 * 1e3);
    }
    CK(hipDeviceSynchronize());
    return 0;
}
