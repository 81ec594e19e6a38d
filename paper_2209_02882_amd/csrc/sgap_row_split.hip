// Row-split schedule: the unit of work is a row of A (the paper's second
// atomic-parallelism family, <x row, y col>, Section 3.2).  Every row is
// produced by exactly one group (parallel strategy) or one lane (serial
// strategy), so results are written with plain stores and empty rows are
// written as zeros by their owner; no atomics, no zero-fill pass.
#include "sgap_common.hpp"
#include "sgap_lane_ops.hpp"

namespace sgap {

// {<1/g row, c col>, r} with g = r = G (Section 6.2, the "1/g row" listing):
// G lanes share a row, lane `member` takes the row's entries member,
// member+G, ... serially, then the group tree-sums and member 0 stores.
//   lane = (slot*G + member)*LC + chunk ; one slot = one row
template <int G, int LC, int VEC>
__global__ __launch_bounds__(kBlock) void row_split_parallel_kernel(SpmmArgs a)
{
    constexpr int SPAN = G * LC;
    constexpr int ROWS_PER_WAVE = kWave / SPAN;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int slot = lane / SPAN;
    const int member = (lane / LC) % G;
    const int chunk = lane % LC;

    const int64_t row = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * ROWS_PER_WAVE + slot;
    const bool row_ok = row < a.M;
    uint32_t p_begin = 0, p_end = 0;
    if (row_ok) {
        p_begin = (uint32_t)a.rowptr[row];
        p_end = (uint32_t)a.rowptr[row + 1];
    }
    const int64_t N = a.N;

    // column tiles of LC*VEC columns; the trip count is uniform over the wave
    for (int64_t k0 = 0; k0 < N; k0 += (int64_t)LC * VEC) {
        const int64_t k = k0 + (int64_t)chunk * VEC;
        const bool k_ok = k < N;
        Vec<VEC> acc;
        acc.zero();
        if (k_ok) {
            const float* __restrict__ Bk = a.B + k;
            uint32_t p = p_begin + member;
            // two entries in flight per lane
            for (; p + G < p_end; p += 2 * G) {
                const int32_t c0 = a.colidx[p];
                const int32_t c1 = a.colidx[p + G];
                const float v0 = a.vals[p];
                const float v1 = a.vals[p + G];
                const Vec<VEC> b0 = load_vec<VEC>(Bk + (int64_t)c0 * N);
                const Vec<VEC> b1 = load_vec<VEC>(Bk + (int64_t)c1 * N);
                acc.fma(v0, b0);
                acc.fma(v1, b1);
            }
            if (p < p_end) {
                const int32_t c0 = a.colidx[p];
                const float v0 = a.vals[p];
                acc.fma(v0, load_vec<VEC>(Bk + (int64_t)c0 * N));
            }
        }
        // lanes without work contributed +0 (zero extension); all lanes reduce
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc.v[i] = group_tree_sum<G, LC>(acc.v[i]);
        if (member == 0 && row_ok && k_ok) store_vec<VEC>(a.C + row * N + k, acc);
    }
}

// {<g row, c col>, 1} (Section 6.1, the "g row" listing): reduction
// parallelism 1.  A lane owns `group` consecutive rows for its column chunk
// and walks each row serially.
//   lane = row_lane*LC + chunk
template <int LC, int VEC>
__global__ __launch_bounds__(kBlock) void row_split_serial_kernel(SpmmArgs a)
{
    constexpr int ROW_LANES = kWave / LC;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_lane = lane / LC;
    const int chunk = lane % LC;
    const int64_t N = a.N;
    const int64_t row0 = (((int64_t)blockIdx.x * kWavesPerBlock + wave) * ROW_LANES + row_lane) * a.group;
    const int64_t row1 = row0 + a.group < a.M ? row0 + a.group : a.M;

    for (int64_t k0 = 0; k0 < N; k0 += (int64_t)LC * VEC) {
        const int64_t k = k0 + (int64_t)chunk * VEC;
        if (k >= N) continue;
        const float* __restrict__ Bk = a.B + k;
        for (int64_t row = row0; row < row1; ++row) {
            uint32_t p = (uint32_t)a.rowptr[row];
            const uint32_t p_end = (uint32_t)a.rowptr[row + 1];
            Vec<VEC> acc;
            acc.zero();
            for (; p + 1 < p_end; p += 2) {
                const int32_t c0 = a.colidx[p];
                const int32_t c1 = a.colidx[p + 1];
                const float v0 = a.vals[p];
                const float v1 = a.vals[p + 1];
                const Vec<VEC> b0 = load_vec<VEC>(Bk + (int64_t)c0 * N);
                const Vec<VEC> b1 = load_vec<VEC>(Bk + (int64_t)c1 * N);
                acc.fma(v0, b0);
                acc.fma(v1, b1);
            }
            if (p < p_end) acc.fma(a.vals[p], load_vec<VEC>(Bk + (int64_t)a.colidx[p] * N));
            store_vec<VEC>(a.C + row * N + k, acc);
        }
    }
}

namespace {
struct LaunchRowSplitParallel {
    const SpmmArgs& a;
    hipStream_t s;
    template <int G, int LC, int VEC>
    void operator()() const
    {
        constexpr int rows_per_block = kWavesPerBlock * (kWave / (G * LC));
        const int64_t grid = (a.M + rows_per_block - 1) / rows_per_block;
        hipLaunchKernelGGL((row_split_parallel_kernel<G, LC, VEC>), dim3((unsigned)grid), dim3(kBlock), 0, s, a);
    }
};
struct LaunchRowSplitSerial {
    const SpmmArgs& a;
    hipStream_t s;
    template <int G, int LC, int VEC>
    void operator()() const
    {
        const int64_t rows_per_block = (int64_t)kWavesPerBlock * (kWave / LC) * a.group;
        const int64_t grid = (a.M + rows_per_block - 1) / rows_per_block;
        hipLaunchKernelGGL((row_split_serial_kernel<LC, VEC>), dim3((unsigned)grid), dim3(kBlock), 0, s, a);
    }
};
}  // namespace

hipError_t launch_row_split_parallel(const SpmmArgs& a, int lc, int vec, hipStream_t s)
{
    if (!dispatch_group(a.group, lc, vec, LaunchRowSplitParallel{a, s})) return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_row_split_serial(const SpmmArgs& a, int lc, int vec, hipStream_t s)
{
    // group is a run-time loop count here; dispatch on (lc, vec) only
    if (!dispatch_lc<1>(lc, vec, LaunchRowSplitSerial{a, s})) return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace sgap
