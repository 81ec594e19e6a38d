// Nnz-balanced schedule: the row-zeroing pass, the plan (tile size, merge mode)
// of the parallel strategy and the dispatch of its launch to the translation
// units that hold the kernel instances.
#include "sgap_common.hpp"
#include "sgap_nnz_common.hpp"

namespace sgap {

// Rows that will receive global atomic adds (their positions straddle an
// aligned merge block of 2^merge_log2 positions) and rows without stored
// entries are set to +0; merge_log2 < 0: every row is.
// thread = (row_lane, chunk); chunk lanes stride over the row's columns.
template <int VEC>
__global__ __launch_bounds__(kBlock) void zero_rows_kernel(SpmmArgs a, int lcz, int merge_log2)
{
    const int chunk = threadIdx.x % lcz;
    const int row_lane = threadIdx.x / lcz;
    const int rows_per_block = kBlock / lcz;
    const int64_t row = (int64_t)blockIdx.x * rows_per_block + row_lane;
    if (row >= a.M) return;
    const int32_t p_begin = a.rowptr[row];
    const int32_t p_end = a.rowptr[row + 1];
    const bool plain = merge_log2 >= 0 && p_end > p_begin && (p_begin >> merge_log2) == ((p_end - 1) >> merge_log2);
    if (plain) return;
    Vec<VEC> z;
    z.zero();
    float* __restrict__ dst = a.C + row * a.N;
    for (int64_t k = (int64_t)chunk * VEC; k < a.N; k += (int64_t)lcz * VEC) store_vec<VEC>(dst + k, z);
}

NnzPlan plan_nnz_parallel(int group, int lc, int vec)
{
    NnzPlan p;
    // one step covers 4*64/lc positions, kParDepth steps are issued together:
    // at most 1024 positions, so one tile size serves every layout
    p.tile = kParTile;
    const int nslots = p.tile / group + 1;
    p.merge = nslots * (lc * vec * 4 + 8) <= kMergeLdsBudget;
    p.lc = lc;
    // Most of the LDS, and if need be narrower passes: for G = 1 (else a global atomic add per stored entry:
    // stencil27 32 ms against 20 ms, rmat 43 against 10) and for narrow passes (rmat, N = 32, G = 2 and 4:
    // 23 and 10 ms against 6.0 and 3.4).  Wider passes of G >= 2 do better with their few global atomics per
    // row than with one or two resident workgroups per compute unit (stencil27, N = 128, G = 2 and 4: 6.4 and
    // 4.1 ms against 12.1 and 9.3; skewed, N = 256, G = 4: 30 against 39).
    if (!p.merge && (group == 1 || lc * vec <= 32)) {
        int lanes = lc;
        while (nslots * (lanes * vec * 4 + 8) > kMergeLdsLimit && lanes > 1) lanes /= 2;
        if (nslots * (lanes * vec * 4 + 8) <= kMergeLdsLimit) {
            p.lc = lanes;
            p.merge = true;
        }
    }
    int lg = 0;
    while ((1 << lg) < (p.merge ? p.tile : group)) ++lg;
    p.merge_log2 = lg;
    return p;
}

// per-group-size launchers, defined in sgap_nnz_parallel_g*.hip
hipError_t launch_nnz_parallel_g1(const SpmmArgs&, int, int, int, int64_t, bool, hipStream_t);
hipError_t launch_nnz_parallel_g2(const SpmmArgs&, int, int, int, int64_t, bool, hipStream_t);
hipError_t launch_nnz_parallel_g4_16(const SpmmArgs&, int, int, int, int64_t, bool, hipStream_t);
hipError_t launch_nnz_parallel_g8_32_64(const SpmmArgs&, int, int, int, int64_t, bool, hipStream_t);

hipError_t launch_nnz_parallel(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, hipStream_t s)
{
    const NnzPlan plan = plan_nnz_parallel(a.group, lc, vec);
    lc = plan.lc;
    switch (a.group) {
        case 1: return launch_nnz_parallel_g1(a, lc, vec, compute_units, nnz_hint, plan.merge, s);
        case 2: return launch_nnz_parallel_g2(a, lc, vec, compute_units, nnz_hint, plan.merge, s);
        case 4: case 16: return launch_nnz_parallel_g4_16(a, lc, vec, compute_units, nnz_hint, plan.merge, s);
        case 8: case 32: case 64: return launch_nnz_parallel_g8_32_64(a, lc, vec, compute_units, nnz_hint, plan.merge, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_nnz_zero_rows(const SpmmArgs& a, int vec, int merge_log2, hipStream_t s)
{
    int64_t chunks = (a.N + vec - 1) / vec;
    int lcz = 1;
    while (lcz < 64 && lcz < chunks) lcz *= 2;
    const int rows_per_block = kBlock / lcz;
    const int64_t grid = (a.M + rows_per_block - 1) / rows_per_block;
    switch (vec) {
        case 4: hipLaunchKernelGGL((zero_rows_kernel<4>), dim3((unsigned)grid), dim3(kBlock), 0, s, a, lcz, merge_log2); break;
        case 2: hipLaunchKernelGGL((zero_rows_kernel<2>), dim3((unsigned)grid), dim3(kBlock), 0, s, a, lcz, merge_log2); break;
        case 1: hipLaunchKernelGGL((zero_rows_kernel<1>), dim3((unsigned)grid), dim3(kBlock), 0, s, a, lcz, merge_log2); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sgap
