// Row-split kernel template and its launcher; included by the translation
// units that instantiate it (sgap_row_split.hip: one group per row, plain
// stores; sgap_row_split_partial.hip: sub-groups merged with atomics).
#pragma once
#include "sgap_common.hpp"
#include "sgap_gather.hpp"
#include "sgap_lane_ops.hpp"

namespace sgap {

constexpr int kStageCap = 2048;  // (column, value) pairs per LDS chunk: 16 KB
constexpr int kRowCap = 1024;    // rowptr entries kept in LDS per row block (+1)
constexpr int kRowSplitMaxBlock = 512;  // threads per workgroup: 128, 256 or 512, chosen at launch

// PARTIAL: the G members of a row reduce in sub-groups of `reduce_members`
// (a power of two below G) and the first member of every sub-group adds its
// sum to C with atomics; C must hold zeros before the launch.
// SKIP: leave the rows described by `skip` alone.
// The workgroup size (the paper's blockSz, Section 7.2) is the launch's: SLOTS = blockDim.x / (G*LC)
// groups work side by side on the rows of a row block.
template <int G, int LC, int VEC, bool OFF32, bool PARTIAL, bool SKIP = false>
__global__ __launch_bounds__(kRowSplitMaxBlock) void row_split_kernel(SpmmArgs a, TileSched ts, int rows_per_slot,
                                                                      int interleave, int reduce_members, RowSkip skip)
{
    __shared__ StagedEntry s_A[kStageCap];
    __shared__ int32_t s_rp[kRowCap + 1];
    constexpr int SPAN = G * LC;
    const int block = blockDim.x;
    const int SLOTS = block / SPAN;

    const int slot = threadIdx.x / SPAN;
    const int member = (threadIdx.x / LC) % G;
    const int chunk = threadIdx.x % LC;
    const int64_t N = a.N;
    const int64_t rows_per_block = (int64_t)SLOTS * rows_per_slot;
    const bool rp_in_lds = rows_per_block <= kRowCap;
    bool skip_on = false;
    if constexpr (SKIP) skip_on = *skip.count <= skip.max_rows;

    // persistent walk over this die's run of work items
    const int64_t xcd = blockIdx.x % ts.xcds;
    const int64_t wg_in_xcd = blockIdx.x / ts.xcds;
    const int64_t wgs_per_xcd = gridDim.x / ts.xcds;
    for (int64_t it = wg_in_xcd; it < ts.items_per_xcd; it += wgs_per_xcd) {
        const int64_t item = xcd * ts.items_per_xcd + it;
        if (item >= ts.items) break;
        const int32_t col_tile = (int32_t)(item / ts.row_blocks);
        const int64_t row_block = item % ts.row_blocks;

        const int64_t row_first = row_block * rows_per_block;
        const int64_t row_last = row_first + rows_per_block < a.M ? row_first + rows_per_block : a.M;
        // this slot's rows, counted from row_first: my_first, my_first + row_step, ... below my_last
        // (32-bit: a row block has at most SLOTS * rows_per_slot rows)
        const int32_t block_rows = (int32_t)(row_last - row_first);
        const int32_t row_step = interleave ? SLOTS : 1;
        int32_t my_first = interleave ? slot : slot * rows_per_slot;
        int32_t my_last = interleave ? block_rows : my_first + rows_per_slot;
        if (my_first > block_rows) my_first = block_rows;
        if (my_last > block_rows) my_last = block_rows;

        __syncthreads();  // everyone is done with the previous item's LDS contents
        if (rp_in_lds) {
            for (int i = threadIdx.x; i <= block_rows; i += block)
                s_rp[i] = a.rowptr[row_first + i];
            __syncthreads();
        }
        const uint32_t nz_first = (uint32_t)a.rowptr[row_first];
        const uint32_t nz_last = (uint32_t)a.rowptr[row_last];

        const int64_t k_tile_end =
            (int64_t)(col_tile + 1) * ts.tile_cols < N ? (int64_t)(col_tile + 1) * ts.tile_cols : N;
        // a tile may be wider than one pass of the LC chunk lanes
        for (int64_t k0 = (int64_t)col_tile * ts.tile_cols; k0 < k_tile_end; k0 += (int64_t)LC * VEC) {
            const int32_t k = (int32_t)k0 + chunk * VEC;  // N < 2^31
            const bool k_ok = k < k_tile_end;
            const GlobalRows<VEC, OFF32> Brow(a.B, N, k);

            int32_t row = my_first;
            Vec<VEC> acc;
            acc.zero();
            for (uint32_t base = nz_first;; base += kStageCap) {  // runs at least once: empty rows get stored
                const uint32_t cnt = nz_last - base < (uint32_t)kStageCap ? nz_last - base : (uint32_t)kStageCap;
                if (base != nz_first || k0 != (int64_t)col_tile * ts.tile_cols) __syncthreads();
                stage_entries(a, base, cnt, s_A, block);
                __syncthreads();
                // rows of this slot that have entries in the chunk (or are empty)
                while (row < my_last) {
                    uint32_t p_begin, p_end;
                    if (rp_in_lds) {
                        p_begin = (uint32_t)s_rp[row];
                        p_end = (uint32_t)s_rp[row + 1];
                    } else {
                        p_begin = (uint32_t)a.rowptr[row_first + row];
                        p_end = (uint32_t)a.rowptr[row_first + row + 1];
                    }
                    const uint32_t lo = p_begin > base ? p_begin : base;
                    const uint32_t hi = p_end < base + cnt ? p_end : base + cnt;
                    bool skipped = false;
                    if constexpr (SKIP) skipped = skip_on && p_end - p_begin >= (uint32_t)skip.min_len;
                    if (!skipped && k_ok && lo < hi) {
                        // first position >= lo that belongs to this member
                        const uint32_t first = lo + ((member - (lo - p_begin)) & (G - 1));
                        if (first < hi) gather_fma<VEC, G>(acc, s_A, first - base, hi - base, Brow);
                    }
                    if (p_end > base + cnt) break;  // the row continues in the next chunk
                    // members without entries contributed +0 (zero extension);
                    // the lanes of a slot reach this point together
                    if constexpr (PARTIAL) {
#pragma unroll
                        for (int i = 0; i < VEC; ++i)
                            acc.v[i] = group_partial_sum<G, LC>(acc.v[i], reduce_members * LC);
                        // a sub-group whose first member has no entry of the row holds +0
                        const bool adds = (member & (reduce_members - 1)) == 0 && (uint32_t)member < p_end - p_begin;
                        if constexpr (LC >= VEC) {
                            // The LC chunk lanes of a member hold LC*VEC consecutive columns, VEC per
                            // lane.  An atomic instruction whose lanes are 16 bytes apart costs four
                            // times one over consecutive words (451 against 115 clocks of the memory
                            // pipeline, measured), so the sums change hands first: in round q lane c
                            // adds column q*LC + c, which lane (q*LC + c) / VEC of the member holds.
#pragma unroll
                            for (int q = 0; q < VEC; ++q) {
                                const int col = q * LC + chunk;
                                float mine = 0.0f;
#pragma unroll
                                for (int v = 0; v < VEC; ++v) {
                                    const float t = __shfl(acc.v[v], col / VEC, LC);
                                    if (col % VEC == v) mine = t;
                                }
                                if (adds && k0 + col < k_tile_end)
                                    unsafeAtomicAdd(a.C + (row_first + row) * N + k0 + col, mine);
                            }
                        } else {
                            if (adds && k_ok) atomic_add_vec<VEC>(a.C + (row_first + row) * N + k, acc);
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < VEC; ++i) acc.v[i] = group_tree_sum<G, LC>(acc.v[i]);
                        if (member == 0 && k_ok && !skipped) store_vec_stream<VEC>(a.C + (row_first + row) * N + k, acc);
                    }
                    acc.zero();
                    row += row_step;
                }
                if (base + cnt >= nz_last) break;
            }
        }
    }
}

namespace row_split_detail {

template <bool PARTIAL, bool SKIP = false>
struct Launch {
    const SpmmArgs& a;
    int rows_per_slot, interleave, tile_cols, xcds, compute_units;
    bool off32, persistent;
    int reduce_members;
    int block;  // threads per workgroup: 128, 256 or 512 (at least G*LC)
    hipStream_t s;
    RowSkip skip = {nullptr, 0, 0};

    // workgroups of this instance that one compute unit can hold at once
    template <typename K>
    static int resident_per_cu(K kernel, int block)
    {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, block, 0) != hipSuccess || n < 1) n = 1;
        return n;
    }

    template <int G, int LC, int VEC>
    void operator()() const
    {
        // a persistent grid must be resident all at once (asked of the runtime only for such launches)
        int max_grid = 0x7fffffff;
        if (persistent)
            max_grid = compute_units * (off32 ? resident_per_cu(row_split_kernel<G, LC, VEC, true, PARTIAL, SKIP>, block)
                                              : resident_per_cu(row_split_kernel<G, LC, VEC, false, PARTIAL, SKIP>, block));
        const int slots = block / (G * LC);
        const int64_t rows_per_block = (int64_t)slots * rows_per_slot;
        TileSched ts;
        ts.row_blocks = (a.M + rows_per_block - 1) / rows_per_block;
        ts.tile_cols = tile_cols;
        ts.col_tiles = (int32_t)((a.N + tile_cols - 1) / tile_cols);
        ts.items = ts.row_blocks * ts.col_tiles;
        ts.xcds = xcds;
        ts.items_per_xcd = (ts.items + xcds - 1) / xcds;
        int64_t wgs_per_xcd = max_grid / xcds > 0 ? max_grid / xcds : 1;
        if (wgs_per_xcd * xcds > 0x7ffffff0LL) wgs_per_xcd = 0x7ffffff0LL / xcds;
        if (wgs_per_xcd > ts.items_per_xcd) wgs_per_xcd = ts.items_per_xcd;
        const unsigned grid = (unsigned)(wgs_per_xcd * xcds);
        if (off32)
            hipLaunchKernelGGL((row_split_kernel<G, LC, VEC, true, PARTIAL, SKIP>), dim3(grid), dim3(block), 0, s, a,
                               ts, rows_per_slot, interleave, reduce_members, skip);
        else
            hipLaunchKernelGGL((row_split_kernel<G, LC, VEC, false, PARTIAL, SKIP>), dim3(grid), dim3(block), 0, s, a,
                               ts, rows_per_slot, interleave, reduce_members, skip);
    }
};

}  // namespace row_split_detail

}  // namespace sgap
