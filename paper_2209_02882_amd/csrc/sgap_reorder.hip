// Row order: an optional preprocessing pass that writes a copy of a CSR matrix whose rows are grouped by a
// coarse key.  The schedules of Section 6 take the rows in the order in which they are stored, and what a
// wavefront's lanes meet there decides how well they run together; Section 2.2 names the line of work on
// locality and balance that a better order stands for.  The product comes out in the new row order: row j of
// C = A' * B is row perm[j] of A * B.
//
// Keys (kOrderBuckets of them, smaller key first, any order inside a key):
//   by first column: bucket of the row's first stored column, K columns cut into equal bucket ranges; rows
//     without entries come last.  Rows that start in the same range of B meet in time.
//   by length: longest rows first (all rows of at least kOrderBuckets - 1 entries share the first key), rows
//     without entries last.  Lanes of a wavefront then walk rows of one length, and the runs of rows without
//     entries no longer lie between the others.
// What it buys where it was measured (R-MAT, 2 M rows, 44 % of them without entries, nnz-balanced serial
// schedule): 0.96 -> 0.71 ms with either key, at the SAME bytes fetched from HBM and 14 % fewer vector
// instructions: the gain is in how alike the lanes' work is, not in cache reuse.  (Moving only the rows
// without entries to the end gives 0.85 ms.)  A stencil in its natural order and uniform random columns gain
// nothing.
// A bucket sort in three steps: every workgroup counts its rows per key in LDS and takes a run of places per
// key from the global counters with one returning atomic per key it holds (a returning atomic per row on a
// counter that a million rows share would take a tenth of a second); the counters are summed up; every row
// goes to the start of its key's run plus its place within the key.
#include "sgap_common.hpp"

namespace sgap {

constexpr int kOrderBuckets = 4097;                  // keys 0 .. 4096
constexpr int kOrderRowsPerThread = 8;
constexpr int kOrderRowsPerBlock = kBlock * kOrderRowsPerThread;

struct OrderView {
    int32_t* key;     // M
    int32_t* within;  // M: place of the row among the rows of its key
    uint32_t* count;  // kOrderBuckets: rows per key
    uint32_t* start;  // kOrderBuckets: first place of a key's run
    int32_t* sums;    // one per block of kOrderRowsPerBlock rows (entries of the block's rows, new order)
};

int64_t reorder_workspace_bytes(int64_t M)
{
    const int64_t blocks = (M + kOrderRowsPerBlock - 1) / kOrderRowsPerBlock + 1;
    const int64_t bytes = 8 * M + 8 * (int64_t)kOrderBuckets + 4 * blocks;
    return (bytes + 255) / 256 * 256 + 256;
}

namespace {

OrderView order_view(void* workspace, int64_t M)
{
    OrderView v;
    char* base = static_cast<char*>(workspace);
    v.key = reinterpret_cast<int32_t*>(base);
    v.within = v.key + M;
    v.count = reinterpret_cast<uint32_t*>(v.within + M);
    v.start = v.count + kOrderBuckets;
    v.sums = reinterpret_cast<int32_t*>(v.start + kOrderBuckets);
    return v;
}

__device__ __forceinline__ int32_t order_key(int64_t K, const int32_t* __restrict__ rowptr,
                                             const int32_t* __restrict__ colidx, int64_t row, int by_length)
{
    const int32_t p0 = rowptr[row], p1 = rowptr[row + 1];
    if (p1 <= p0) return kOrderBuckets - 1;
    if (by_length) {
        const int32_t len = p1 - p0;
        return len >= kOrderBuckets - 1 ? 0 : kOrderBuckets - 1 - len;
    }
    int64_t key = (int64_t)colidx[p0] * (kOrderBuckets - 1) / K;  // 0 .. kOrderBuckets - 2 for a column inside [0, K)
    if (key < 0) key = 0;                                          // (a column outside must not index past the counters)
    if (key > kOrderBuckets - 2) key = kOrderBuckets - 2;
    return (int32_t)key;
}

// Exclusive prefix sum over the workgroup's threads (thread order); *total = the sum over all of them.
__device__ __forceinline__ int32_t block_exclusive_sum(int32_t v, int32_t* total, int32_t* s_wave)
{
    const int lane = threadIdx.x % kWave;
    const int wave = threadIdx.x / kWave;
    int32_t incl = v;
#pragma unroll
    for (int d = 1; d < kWave; d *= 2) {
        const int32_t t = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += t;
    }
    __syncthreads();  // s_wave may still be read from an earlier call
    if (lane == kWave - 1) s_wave[wave] = incl;
    __syncthreads();
    int32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
        const int32_t c = s_wave[w];
        if (w < wave) before += c;
        all += c;
    }
    *total = all;
    return before + incl - v;
}

}  // namespace

__global__ void order_reset_kernel(OrderView v)
{
    for (int b = threadIdx.x; b < kOrderBuckets; b += blockDim.x) v.count[b] = 0;
}

__global__ __launch_bounds__(kBlock) void order_count_kernel(int64_t M, int64_t K, const int32_t* __restrict__ rowptr,
                                                             const int32_t* __restrict__ colidx, int by_length,
                                                             OrderView v)
{
    __shared__ uint32_t s_count[kOrderBuckets];  // rows per key in this workgroup, then the workgroup's first place
    for (int b = threadIdx.x; b < kOrderBuckets; b += kBlock) s_count[b] = 0;
    __syncthreads();
    const int64_t row0 = (int64_t)blockIdx.x * kOrderRowsPerBlock + threadIdx.x;
    int32_t key[kOrderRowsPerThread];
    uint32_t place[kOrderRowsPerThread];
#pragma unroll
    for (int j = 0; j < kOrderRowsPerThread; ++j) {
        const int64_t row = row0 + (int64_t)j * kBlock;
        key[j] = -1;
        place[j] = 0;
        if (row < M) {
            key[j] = order_key(K, rowptr, colidx, row, by_length);
            place[j] = atomicAdd(&s_count[key[j]], 1u);
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < kOrderBuckets; b += kBlock) {
        const uint32_t c = s_count[b];
        if (c) s_count[b] = atomicAdd(&v.count[b], c);
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kOrderRowsPerThread; ++j) {
        const int64_t row = row0 + (int64_t)j * kBlock;
        if (row < M) {
            v.key[row] = key[j];
            v.within[row] = (int32_t)(s_count[key[j]] + place[j]);
        }
    }
}

// start[b] = rows with a smaller key (one workgroup)
__global__ __launch_bounds__(kBlock) void order_starts_kernel(OrderView v)
{
    __shared__ int32_t s_wave[kWavesPerBlock];
    constexpr int PER = (kOrderBuckets + kBlock - 1) / kBlock;
    const int b0 = threadIdx.x * PER;
    int32_t mine = 0;
    for (int j = 0; j < PER; ++j)
        if (b0 + j < kOrderBuckets) mine += (int32_t)v.count[b0 + j];
    int32_t total;
    int32_t run = block_exclusive_sum(mine, &total, s_wave);
    for (int j = 0; j < PER; ++j) {
        if (b0 + j >= kOrderBuckets) break;
        v.start[b0 + j] = (uint32_t)run;
        run += (int32_t)v.count[b0 + j];
    }
}

__global__ __launch_bounds__(kBlock) void order_place_kernel(int64_t M, OrderView v, int32_t* __restrict__ perm)
{
    const int64_t row = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (row < M) perm[v.start[v.key[row]] + (uint32_t)v.within[row]] = (int32_t)row;
}

// Stored entries of the rows of one block of kOrderRowsPerBlock rows, new order.
__global__ __launch_bounds__(kBlock) void order_block_sums_kernel(int64_t M, const int32_t* __restrict__ rowptr,
                                                                  const int32_t* __restrict__ perm, OrderView v)
{
    __shared__ int32_t s_wave[kWavesPerBlock];
    const int64_t j0 = (int64_t)blockIdx.x * kOrderRowsPerBlock + (int64_t)threadIdx.x * kOrderRowsPerThread;
    int32_t mine = 0;
#pragma unroll
    for (int u = 0; u < kOrderRowsPerThread; ++u) {
        if (j0 + u < M) {
            const int32_t row = perm[j0 + u];
            mine += rowptr[row + 1] - rowptr[row];
        }
    }
    int32_t total;
    (void)block_exclusive_sum(mine, &total, s_wave);
    if (threadIdx.x == 0) v.sums[blockIdx.x] = total;
}

// sums[] -> entries in front of each block (one workgroup)
__global__ __launch_bounds__(kBlock) void order_scan_sums_kernel(int64_t blocks, OrderView v)
{
    __shared__ int32_t s_wave[kWavesPerBlock];
    int32_t carry = 0;
    for (int64_t base = 0; base < blocks; base += kBlock) {
        const int64_t b = base + threadIdx.x;
        const int32_t mine = b < blocks ? v.sums[b] : 0;
        int32_t total;
        const int32_t before = block_exclusive_sum(mine, &total, s_wave);
        if (b < blocks) v.sums[b] = carry + before;
        carry += total;
    }
}

__global__ __launch_bounds__(kBlock) void order_rowptr_kernel(int64_t M, const int32_t* __restrict__ rowptr,
                                                              const int32_t* __restrict__ perm, OrderView v,
                                                              int32_t* __restrict__ rowptr_out)
{
    __shared__ int32_t s_wave[kWavesPerBlock];
    const int64_t j0 = (int64_t)blockIdx.x * kOrderRowsPerBlock + (int64_t)threadIdx.x * kOrderRowsPerThread;
    int32_t len[kOrderRowsPerThread];
    int32_t mine = 0;
#pragma unroll
    for (int u = 0; u < kOrderRowsPerThread; ++u) {
        len[u] = 0;
        if (j0 + u < M) {
            const int32_t row = perm[j0 + u];
            len[u] = rowptr[row + 1] - rowptr[row];
        }
        mine += len[u];
    }
    int32_t total;
    int32_t run = v.sums[blockIdx.x] + block_exclusive_sum(mine, &total, s_wave);
#pragma unroll
    for (int u = 0; u < kOrderRowsPerThread; ++u) {
        if (j0 + u < M) rowptr_out[j0 + u] = run;
        run += len[u];
        if (j0 + u == M - 1) rowptr_out[M] = run;
    }
}

// One wavefront per row of the new matrix copies the row's entries.
__global__ __launch_bounds__(kBlock) void order_copy_rows_kernel(int64_t M, const int32_t* __restrict__ rowptr,
                                                                 const int32_t* __restrict__ colidx,
                                                                 const float* __restrict__ vals,
                                                                 const int32_t* __restrict__ perm,
                                                                 const int32_t* __restrict__ rowptr_out,
                                                                 int32_t* __restrict__ colidx_out,
                                                                 float* __restrict__ vals_out)
{
    const int lane = threadIdx.x % kWave;
    const int64_t waves = (int64_t)gridDim.x * kWavesPerBlock;
    for (int64_t j = (int64_t)blockIdx.x * kWavesPerBlock + threadIdx.x / kWave; j < M; j += waves) {
        const int32_t row = perm[j];
        const int32_t src = rowptr[row];
        const int32_t len = rowptr[row + 1] - src;
        const int32_t dst = rowptr_out[j];
        for (int32_t q = lane; q < len; q += kWave) {
            colidx_out[dst + q] = colidx[src + q];
            vals_out[dst + q] = vals[src + q];
        }
    }
}

hipError_t launch_reorder_rows(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colidx, const float* vals,
                               bool by_length, int32_t* perm, int32_t* rowptr_out, int32_t* colidx_out,
                               float* vals_out, void* workspace, int compute_units, hipStream_t s)
{
    const OrderView v = order_view(workspace, M);
    const unsigned blocks = (unsigned)((M + kOrderRowsPerBlock - 1) / kOrderRowsPerBlock);
    hipLaunchKernelGGL(order_reset_kernel, dim3(1), dim3(kBlock), 0, s, v);
    hipLaunchKernelGGL(order_count_kernel, dim3(blocks), dim3(kBlock), 0, s, M, K, rowptr, colidx, by_length ? 1 : 0, v);
    hipLaunchKernelGGL(order_starts_kernel, dim3(1), dim3(kBlock), 0, s, v);
    hipLaunchKernelGGL(order_place_kernel, dim3((unsigned)((M + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, M, v, perm);
    hipLaunchKernelGGL(order_block_sums_kernel, dim3(blocks), dim3(kBlock), 0, s, M, rowptr, perm, v);
    hipLaunchKernelGGL(order_scan_sums_kernel, dim3(1), dim3(kBlock), 0, s, (int64_t)blocks, v);
    hipLaunchKernelGGL(order_rowptr_kernel, dim3(blocks), dim3(kBlock), 0, s, M, rowptr, perm, v, rowptr_out);
    int64_t grid = (int64_t)compute_units * 8;
    const int64_t needed = (M + kWavesPerBlock - 1) / kWavesPerBlock;
    if (grid > needed) grid = needed;
    hipLaunchKernelGGL(order_copy_rows_kernel, dim3((unsigned)grid), dim3(kBlock), 0, s, M, rowptr, colidx, vals, perm,
                       rowptr_out, colidx_out, vals_out);
    return hipGetLastError();
}

}  // namespace sgap
