// Microbenchmark behind the choice of how partial sums are merged in LDS:
// throughput of the LDS fp32 atomic add against integer LDS atomics, plain LDS
// stores and a compare-and-swap loop that adds floats on the integer path, all
// on conflict-free addresses.  Standalone: hipcc --offload-arch=gfx950 -O3 lds_atomics.hip
#include <hip/hip_runtime.h>
#include <cstdio>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
template <int MODE>
__global__ __launch_bounds__(256) void k(float* out, int iters)
{
    __shared__ float s[256 * 4];
    for (int i = threadIdx.x; i < 1024; i += 256) s[i] = 0.0f;
    __syncthreads();
    const int t = threadIdx.x;
    float v = (float)t;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float* p = s + j * 256 + ((t + it) & 255);   // conflict-free, address changes per iteration
            if (MODE == 0) __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            else if (MODE == 1) __hip_atomic_fetch_add((int*)p, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            else if (MODE == 3) {
                int* ip = (int*)p;
                int old = *(volatile int*)ip;
                while (true) {
                    const int want = __float_as_int(__int_as_float(old) + v);
                    const int seen = atomicCAS(ip, old, want);
                    if (seen == old) break;
                    old = seen;
                }
            }
            else *(volatile float*)p = v;
        }
    }
    __syncthreads();
    out[blockIdx.x * 256 + t] = s[t] + s[256 + t];
}
int main()
{
    float* out; CHECK(hipMalloc(&out, 4096 * 256 * 4));
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    const int iters = 2000, grid = 2048;
    const char* names[4] = {"ds_add_f32", "ds_add_u32", "ds_write_b32", "cas-loop fadd"};
    for (int mode = 0; mode < 4; ++mode) {
        for (int rep = 0; rep < 2; ++rep) {
            CHECK(hipEventRecord(e0));
            if (mode == 0) hipLaunchKernelGGL(k<0>, dim3(grid), dim3(256), 0, 0, out, iters);
            if (mode == 1) hipLaunchKernelGGL(k<1>, dim3(grid), dim3(256), 0, 0, out, iters);
            if (mode == 2) hipLaunchKernelGGL(k<2>, dim3(grid), dim3(256), 0, 0, out, iters);
            if (mode == 3) hipLaunchKernelGGL(k<3>, dim3(grid), dim3(256), 0, 0, out, iters);
            CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
            float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
            double ops = (double)grid * 256 * iters * 4;
            if (rep) printf("%-14s %8.3f ms  %8.1f G lane-ops/s  %6.2f lane-ops/clk/CU (256 CUs, 2.4 GHz)\n", names[mode], ms, ops / ms / 1e6, ops / (ms * 1e-3) / 256 / 2.4e9);
        }
    }
    return 0;
}
