// Microbenchmark behind the gather ceilings quoted for the SpMM kernels: how
// fast can a compute unit gather contiguous segments of 128 B .. 1 KB at
// random rows (16-byte loads per lane, 8 in flight, as the kernels do), as a
// function of the window the rows are drawn from (L1-, L2-, Infinity-Cache-
// and HBM-sized).  Standalone: hipcc --offload-arch=gfx950 -O3 gather_bandwidth.hip
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("err %s line %d\n",hipGetErrorString(e),__LINE__); return 1;}}while(0)

template <int LC>  // lanes per row segment (segment bytes = LC*16)
__global__ __launch_bounds__(256) void gather(const float4* __restrict__ buf, float* out, uint32_t rows, uint32_t row_f4, int iters, uint32_t seed)
{
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t seg = (blockIdx.x * 4 + (threadIdx.x >> 6)) * (64 / LC) + lane / LC;  // global segment-lane id
    const uint32_t chunk = lane % LC;
    float4 acc = make_float4(0,0,0,0);
    uint32_t s = seg * 2654435761u + seed;
    for (int it = 0; it < iters; ++it) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            s = s * 1664525u + 1013904223u;
            const uint32_t r = (uint32_t)(((uint64_t)(s >> 4) * rows) >> 28);
            v[u] = buf[(size_t)r * row_f4 + chunk];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
    if (acc.x + acc.y + acc.z + acc.w == 123.456f) out[0] = acc.x;
}

template <int LC>
int run(const float4* buf, float* out, const char* name, uint32_t rows, uint32_t row_bytes, int blocks_per_cu)
{
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    const int blocks = 256 * blocks_per_cu; const int iters = 400;
    gather<LC><<<blocks, 256>>>(buf, out, rows, row_bytes / 16, 10, 1); CK(hipDeviceSynchronize());
    hipEventRecord(e0);
    gather<LC><<<blocks, 256>>>(buf, out, rows, row_bytes / 16, iters, 7);
    hipEventRecord(e1); CK(hipEventSynchronize(e1));
    float ms; hipEventElapsedTime(&ms, e0, e1);
    double bytes = (double)blocks * 256 * 16 * 8 * iters;
    printf("%-44s seg %4d B  window %8.1f MB  %8.1f GB/s  %5.1f B/clk/CU\n", name, LC * 16, (double)rows * row_bytes / 1e6, bytes / ms / 1e6, bytes / (ms * 1e-3) / 2.4e9 / 256);
    return 0;
}

int main()
{
    float4* buf; float* out;
    size_t total = (size_t)1 << 30;
    CK(hipMalloc(&buf, total)); CK(hipMemset(buf, 0, total)); CK(hipMalloc(&out, 4));
    // row stride 512 B (N=128): windows 64KB(L1-ish) 2MB (L2), 64MB (MALL), 1GB (HBM)
    for (uint32_t rows : {64u, 4096u, 131072u, 2097152u}) {
        run<32>(buf, out, "stride 512B, full row (LC=32)", rows, 512, 8);
        run<8>(buf, out, "stride 512B, 128B segment (LC=8)", rows, 512, 8);
    }
    for (uint32_t rows : {256u, 16384u, 524288u, 8388608u}) run<8>(buf, out, "stride 128B rows (N=32, LC=8)", rows, 128, 8);
    for (uint32_t rows : {32u, 2048u, 65536u, 1048576u}) run<64>(buf, out, "stride 1KB rows (N=256, LC=64)", rows, 1024, 8);
    run<32>(buf, out, "stride 512B full row, 4 blocks/CU", 4096, 512, 4);
    run<32>(buf, out, "stride 512B full row, 2 blocks/CU", 4096, 512, 2);
    return 0;
}
