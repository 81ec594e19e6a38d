// Cross-lane building blocks for wave64 segment groups (gfx950).
//
// A segment group (the paper's Section 4: the unit that carries the
// synchronisation semantics, separate from tiling) is G lanes of one
// wavefront.  Lanes of a wave are laid out as
//     lane = (slot * G + member) * LC + chunk
// i.e. LC neighbouring lanes hold neighbouring column chunks of the dense
// operand (so that a row of B is read as one contiguous run), and the G
// members of a group sit LC lanes apart.  SPAN = G*LC lanes form one slot.
//
// The two primitives are this library's versions of the paper's macro
// instructions (Section 5.3): group_tree_sum for atomicAddGroup<T,G> (all
// members feed one output) and group_seg_sum for segReduceGroup<T,G> (members
// feed the output of their own run of equal rows).  They are written for
// 64-lane wavefronts with DPP row shifts, lane-swap and LDS-crossbar permutes.
#pragma once
#include <hip/hip_runtime.h>

namespace sgap {

__device__ __forceinline__ int lane_id()
{
    return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// DPP move, row_shl:S : lane i receives the value of lane i+S of the same
// row of 16 lanes (0 where that lane does not exist).
template <int S>
__device__ __forceinline__ float dpp_row_shl(float v)
{
    static_assert(S >= 1 && S <= 15, "row shift range");
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x100 + S, 0xF, 0xF, true));
}

// Value of lane i+S through the LDS crossbar (no LDS memory is touched).
// Lanes whose source would be >= 64 wrap around; callers ignore those.
template <int S>
__device__ __forceinline__ float bperm_from_above(float v)
{
    const int src = (lane_id() + S) & 63;
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src << 2, __builtin_bit_cast(int, v)));
}

// One halving step of a tree sum: afterwards every lane in the LOWER half of
// each aligned block of 2*S lanes holds v[i] + v[i+S].
template <int S>
__device__ __forceinline__ float tree_step(float v)
{
    if constexpr (S <= 8) {
        return v + dpp_row_shl<S>(v);
    } else if constexpr (S == 16) {
        // v_permlane16_swap exchanges 16-lane rows between its two operands:
        // with operands (v, 0) the results are [v.row0, 0, v.row2, 0] and
        // [v.row1, 0, v.row3, 0]; their sum is v[i] + v[i+16] in rows 0 and 2.
        auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, v), 0u, false, false);
        const unsigned a = r[0], b = r[1];  // scalars first: bit_cast of a vector element misreads
        return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
    } else {
        static_assert(S == 32, "wave64");
        // same with 32-lane halves: [v.lo, 0] and [v.hi, 0]
        auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, v), 0u, false, false);
        const unsigned a = r[0], b = r[1];
        return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
    }
}

template <int S, int LC>
__device__ __forceinline__ float tree_down(float v)
{
    if constexpr (S >= LC && S >= 1) {
        v = tree_step<S>(v);
        return tree_down<S / 2, LC>(v);
    } else {
        return v;
    }
}

// Sum over the G members of each group (members LC lanes apart).  The result
// is valid in member 0 of the group, for each of its LC chunk lanes.  All 64
// lanes must call this together, outside divergent control flow; lanes with
// nothing to add pass 0 (the paper's "zero extension", Section 5.2).
template <int G, int LC>
__device__ __forceinline__ float group_tree_sum(float v)
{
    static_assert(G * LC <= 64, "a group lives inside one wavefront");
    return tree_down<(G * LC) / 2, LC>(v);
}

template <int S, int LC>
__device__ __forceinline__ float tree_down_below(float v, int limit)
{
    if constexpr (S >= LC && S >= 1) {
        if (S < limit) v = tree_step<S>(v);  // wave-uniform condition
        return tree_down_below<S / 2, LC>(v, limit);
    } else {
        return v;
    }
}

// Sums over sub-groups: the G members of a group reduce in aligned sub-groups
// of R = reduce_lanes / LC members (R a power of two, 1 <= R <= G; reduce_lanes
// is the same in every lane).  The result is valid in the first member of each
// sub-group.  This is the reduction of {<1/g row, c col>, r} with r < g
// (Section 4): the tiling uses G lanes per row, the synchronisation R.
template <int G, int LC>
__device__ __forceinline__ float group_partial_sum(float v, int reduce_lanes)
{
    static_assert(G * LC <= 64, "a group lives inside one wavefront");
    return tree_down_below<(G * LC) / 2, LC>(v, reduce_lanes);
}

// Value of the lane S above, for every lane whose source lies in the same
// aligned block of SPAN lanes.
template <int S, int SPAN>
__device__ __forceinline__ float shift_from_above(float v)
{
    if constexpr (SPAN <= 16) {
        return dpp_row_shl<S>(v);
    } else {
        return bperm_from_above<S>(v);
    }
}

template <int D, int G, int LC>
__device__ __forceinline__ float seg_up(float v, int span)
{
    if constexpr (D < G) {
        const float t = shift_from_above<D * LC, G * LC>(v);
        if (D <= span) v += t;
        return seg_up<D * 2, G, LC>(v, span);
    } else {
        return v;
    }
}

// Segmented sum inside a group.  `span` = number of FOLLOWING members of this
// lane's group that belong to the same run (same output row) as this lane,
// 0 <= span <= G-1-member.  Afterwards every lane holds the sum of its own
// value and the next `span` members' values; the first lane of each run thus
// holds the run total.  Runs are contiguous because rows are non-decreasing
// along the stored entries.  All 64 lanes call together.
template <int G, int LC>
__device__ __forceinline__ float group_seg_sum(float v, int span)
{
    static_assert(G * LC <= 64, "a group lives inside one wavefront");
    return seg_up<1, G, LC>(v, span);
}

}  // namespace sgap
