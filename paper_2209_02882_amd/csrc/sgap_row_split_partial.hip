// Row-split schedule with the tiling and the synchronisation granularity set
// apart: {<1/g row, c col>, r} with r < g (Section 4; the points of Table 1).
// g lanes share a row, every r of them tree-sum, and the g/r sub-group sums of
// a row are merged into C with atomic adds, so C is zeroed first.
#include "sgap_row_split_impl.hpp"

namespace sgap {

hipError_t launch_row_split_partial(const SpmmArgs& a, int g, int r, int lc, int vec, int rows_per_slot,
                                    int tile_cols, int xcds, int compute_units, bool persistent, int block,
                                    hipStream_t s)
{
    if (r < 1 || r >= g || (r & (r - 1)) != 0) return hipErrorInvalidValue;
    row_split_detail::Launch<true> f{a, rows_per_slot, 1, tile_cols, xcds, compute_units,
                                     offsets_fit_32(a), persistent, r, block, s};
    if (!dispatch_group(g, lc, vec, f)) return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace sgap
