// Row-split schedule: the unit of work is a row of A (the paper's second
// atomic-parallelism family, <x row, y col>, Section 3.2).  Every row is
// produced by exactly one group (parallel strategy) or one lane (serial
// strategy), so results are written with plain stores and empty rows are
// written as zeros by their owner; no atomics, no zero-fill pass.
//
// One kernel template serves both strategies:
//   parallel  {<1/g row, c col>, r}, g = r = G (Section 6.2, "1/g row"):
//             the G members of a group share a row; member m takes the row's
//             entries m, m+G, ... serially, the group tree-sums, member 0
//             stores.  A group works through `rows_per_slot` rows of its row
//             block (finite resource parallelism, Section 3.3), interleaved
//             with the other groups' rows so that neighbouring rows, which
//             tend to share columns, are in flight together.
//   serial    {<g row, c col>, 1} (Section 6.1, "g row"): the same kernel with
//             G = 1 and rows_per_slot = group_size.
// Lane layout:  thread = (slot*G + member)*LC + chunk over the workgroup.
//
// A work item is (block of consecutive rows, column tile), one workgroup per
// item (or, as a tuning option, a grid that fits the chip at once whose
// workgroups loop over items); the stored entries of a row block are contiguous in
// colidx/vals, so the workgroup copies them (coalesced, streaming) into LDS in
// chunks together with the block's slice of rowptr, and its lanes then read
// (column, value) pairs from LDS: the vector memory path carries only the
// gathered rows of B.
#include "sgap_row_split_impl.hpp"

namespace sgap {

hipError_t launch_row_split(const SpmmArgs& a, int g, int lc, int vec, int rows_per_slot, bool interleave,
                            int tile_cols, int xcds, int compute_units, bool persistent, int block, hipStream_t s)
{
    row_split_detail::Launch<false> f{a, rows_per_slot, interleave ? 1 : 0, tile_cols, xcds, compute_units,
                                      offsets_fit_32(a), persistent, 0, block, s};
    if (!dispatch_group(g, lc, vec, f)) return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace sgap
