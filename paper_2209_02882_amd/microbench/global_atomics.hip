// Microbenchmark behind the cost model of cross-group merging: throughput of
// global fp32 atomic adds against integer atomics, a compare-and-swap loop and
// plain stores; every wavefront adds to 64 consecutive floats of a random row
// of a 512 MB array.  Two more lines give the fp32 atomic add with the lanes of
// an instruction 16 bytes apart (every fourth float of a 1 KB row) and with
// only 8 of the 64 lanes active, the two shapes a kernel meets when every lane
// owns four consecutive columns or a row is narrow.
// Standalone: hipcc --offload-arch=gfx950 -O3 -munsafe-fp-atomics global_atomics.hip
#include <hip/hip_runtime.h>
#include <cstdio>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)
template <int MODE>
__global__ __launch_bounds__(256) void k(float* buf, size_t n, int iters)
{
    // each wave adds to 64 consecutive floats at a pseudo-random row
    const size_t wave = (size_t)blockIdx.x * 4 + threadIdx.x / 64;
    const int lane = threadIdx.x % 64;
    unsigned h = (unsigned)wave * 2654435761u;
    for (int it = 0; it < iters; ++it) {
        h = h * 1664525u + 1013904223u;
        float* p = buf + ((size_t)(h >> 8) % (n / 64)) * 64 + lane;
        if (MODE == 4) {  // lanes 16 bytes apart: float 4*lane + (it & 3) of a row of 256 floats
            unsafeAtomicAdd(buf + ((size_t)(h >> 8) % (n / 256)) * 256 + 4 * lane + (it & 3), 1.0f);
            continue;
        }
        if (MODE == 5) {  // 8 active lanes, consecutive floats
            if (lane < 8) unsafeAtomicAdd(p, 1.0f);
            continue;
        }
        if (MODE == 0) unsafeAtomicAdd(p, 1.0f);
        else if (MODE == 1) atomicAdd((int*)p, 1);
        else if (MODE == 2) {
            int* ip = (int*)p; int old = __builtin_nontemporal_load(ip);
            while (true) { int want = __float_as_int(__int_as_float(old) + 1.0f); int seen = atomicCAS(ip, old, want); if (seen == old) break; old = seen; }
        } else { *p = 1.0f; }
    }
}
int main()
{
    const size_t n = 128u << 20;  // 512 MB
    float* buf; CHECK(hipMalloc(&buf, n * 4)); CHECK(hipMemset(buf, 0, n * 4));
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    const int iters = 64, grid = 8192;
    const char* names[6] = {"global_atomic_add_f32", "global_atomic_add_i32", "cas-loop fadd", "plain store",
                            "atomic_add_f32, lanes 16 B apart", "atomic_add_f32, 8 lanes"};
    for (int mode = 0; mode < 6; ++mode)
        for (int rep = 0; rep < 2; ++rep) {
            CHECK(hipEventRecord(e0));
            if (mode == 0) hipLaunchKernelGGL(k<0>, dim3(grid), dim3(256), 0, 0, buf, n, iters);
            if (mode == 1) hipLaunchKernelGGL(k<1>, dim3(grid), dim3(256), 0, 0, buf, n, iters);
            if (mode == 2) hipLaunchKernelGGL(k<2>, dim3(grid), dim3(256), 0, 0, buf, n, iters);
            if (mode == 3) hipLaunchKernelGGL(k<3>, dim3(grid), dim3(256), 0, 0, buf, n, iters);
            if (mode == 4) hipLaunchKernelGGL(k<4>, dim3(grid), dim3(256), 0, 0, buf, n, iters);
            if (mode == 5) hipLaunchKernelGGL(k<5>, dim3(grid), dim3(256), 0, 0, buf, n, iters);
            CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
            float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
            double ops = (double)grid * 256 * iters;
            // wavefront instructions per second and compute unit -> clocks at 2.26 GHz under load
            const double instr_per_cu_s = ops / 64 / 256 / (ms * 1e-3);
            if (rep)
                printf("%-34s %8.3f ms  %8.1f G lane-slots/s  %6.0f clocks per wavefront instruction and CU\n", names[mode],
                       ms, ops / ms / 1e6, 2.26e9 / instr_per_cu_s);
        }
    return 0;
}
