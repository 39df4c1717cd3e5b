// Micro-benchmark: sustained LDS read bandwidth per CU for the operand reads the kernels use
// (ds_read_b128, one 16-byte piece per lane, rows 80 / 112 / 144 bytes apart: odd multiples of 16,
// conflict-free) and for ds_read_b32, with 4, 8 and 16 waves per CU.
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops -o lds_read_rate lds_read_rate.hip && ./lds_read_rate
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("err %s line %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)

// Each lane reads `iters` x 8 pieces of W bytes from row (lane % 32) at byte stride `stride`, piece
// index (lane / 32): the access pattern of an MFMA A operand.
template <int W>
__global__ __launch_bounds__(256) void rd(float* out, int iters, int stride, int lds_bytes)
{
    // reads stay below 3 * 4096 + 31 * stride + 32 <= 16 848 bytes; lds_bytes >= 20 480 (checked on the host)
    extern __shared__ __attribute__((aligned(16))) char lds[];
    for (int i = threadIdx.x; i < lds_bytes / 4; i += blockDim.x) ((float*)lds)[i] = (float)i;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const char* base = lds + (wave & 3) * 4096 + (lane & 31) * stride + (lane >> 5) * W;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if (W == 16) {
                float4 v;
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"((uint32_t)(uintptr_t)base), "n"(0));
                asm volatile("s_waitcnt lgkmcnt(7)" ::: "memory");
                acc += v.x;
            } else {
                float v;
                asm volatile("ds_read_b32 %0, %1" : "=v"(v) : "v"((uint32_t)(uintptr_t)base));
                asm volatile("s_waitcnt lgkmcnt(7)" ::: "memory");
                acc += v;
            }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    out[blockIdx.x * blockDim.x + threadIdx.x] = acc;
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
    hipDeviceProp_t prop; CK(hipGetDeviceProperties(&prop, 0));
    const int cus = prop.multiProcessorCount;
    const double ghz = prop.clockRate * 1e-6;
    float* out; CK(hipMalloc(&out, (size_t)cus * 4 * 256 * 4));
    const int iters = 2000;
    printf("%d CUs, %.2f GHz nominal\n", cus, ghz);
    for (int wgs = 1; wgs <= 4; wgs *= 2) {          // 256-lane workgroups per CU: 4, 8, 16 waves
        const int blocks = cus * wgs;
        const int lds_bytes = 32768;                 // 4 workgroups x 32 KB fit the CU's 160 KB
        for (int stride : {80, 112, 144, 128}) {
            float ms = best_ms([&] { rd<16><<<blocks, 256, lds_bytes>>>(out, iters, stride, lds_bytes); });
            double bytes = (double)iters * 8 * 1024 * 4 * wgs;      // per CU
            printf("  %2d waves/CU  ds_read_b128 stride %3d B: %6.1f B/clk/CU (at nominal clock)\n", 4 * wgs, stride,
                   bytes / (ms * 1e-3) / (ghz * 1e9));
        }
        float ms = best_ms([&] { rd<4><<<blocks, 256, lds_bytes>>>(out, iters, 132, lds_bytes); });
        double bytes = (double)iters * 8 * 256 * 4 * wgs;
        printf("  %2d waves/CU  ds_read_b32  stride 132 B: %6.1f B/clk/CU\n", 4 * wgs, bytes / (ms * 1e-3) / (ghz * 1e9));
    }
    CK(hipDeviceSynchronize());
    return 0;
}
