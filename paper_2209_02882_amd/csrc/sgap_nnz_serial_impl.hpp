// Nnz-balanced schedule, serial strategy: {<g nnz, c col>, 1} (Section 6.1,
// the "g nnz" listing).  The unit of work is a stored entry of A; a lane walks
// `group` consecutive stored entries by itself and flushes its register
// whenever the row ends or its share ends (conditional reduction).
//   thread = entry_lane*LC + chunk over the whole workgroup
//
// A workgroup copies a tile of (column, value) pairs into LDS together with
// the window of rowptr the tile touches.  A lane finds the row of its first
// position by searching that window (Listings 1 and 2 search rowptr the same
// way) and then follows the row ends through the window, so the stored
// entries need no per-entry row record.  The loads that bring in the next
// tile are issued before the current tile is multiplied out.
//
// This header holds the kernel templates and the per-layout launcher; it is
// included by the sgap_nnz_serial_lc*.hip translation units, each of which
// instantiates the kernels of a few lane layouts (the instances are split over
// several files only to compile them side by side).
#pragma once
#include "sgap_common.hpp"
#include "sgap_gather.hpp"
#include "sgap_nnz_common.hpp"

namespace sgap {

// Multiply out the chunk [base, end) of the tile staged in s_A (slot s holds
// position tile_start + s), whose rows are s_win[w.n_first .. w.n_last + 1]
// relative to row_lb: window index wi stands for row row_lb + wi, or, when
// s_row is given (a window of the rows WITH entries only), for row s_row[wi].
// MERGE selects tile mode of the merge rule; in that mode the function ends with a barrier.
template <int LC, int VEC, bool OFF32, bool MERGE>
__device__ __forceinline__ void serial_chunk(const SpmmArgs& a, const MergeBuf& mb, const StagedEntry* __restrict__ s_A,
                                             const int32_t* __restrict__ s_win, const RowWindow& w, int32_t row_lb,
                                             int32_t tile_start, int32_t base, int32_t end,
                                             const int32_t* __restrict__ s_row = nullptr)
{
    constexpr int kDepth = 8;  // gathered rows of B in flight per lane
    // How partial sums are added into the LDS slots.  With many chunk lanes per
    // entry a wavefront holds few entry lanes, two or three of which meet on a
    // row's slot: the compare-and-swap loop wins.  With few chunk lanes a
    // wavefront holds up to 64 entry lanes, whole rows of which meet on one
    // slot, and the loop would retry once per lane: the hardware atomic wins
    // (rmat at N=4, one entry per lane: 1.6 ms against 23 ms).
    constexpr bool kCasMerge = LC >= 8;
    constexpr int ENTRY_LANES = kBlock / LC;
    const int entry_lane = threadIdx.x / LC;
    const int chunk = threadIdx.x % LC;
    const int64_t N = a.N;
    const int G = a.group;
    const int per_step = ENTRY_LANES * G;  // positions the workgroup covers per step

    for (int64_t k0 = 0; k0 < N; k0 += (int64_t)LC * VEC) {
        const int64_t k = k0 + (int64_t)chunk * VEC;
        const bool k_ok = k < N;
        const BRow<OFF32> Brow(a.B, N, k);
        for (int32_t blk = tile_start + entry_lane * G; k_ok && blk < end; blk += per_step) {
            // this lane's aligned block of G positions, clipped to the chunk
            const int32_t blk_begin = blk > base ? blk : base;
            const int32_t blk_end = blk + G < end ? blk + G : end;
            if (blk_begin >= blk_end) continue;
            // window index of the row that holds blk_begin
            int32_t wi = last_row_at_or_before(s_win, w.n_first, w.n_last, blk_begin);
            int32_t row_begin = s_win[wi];
            int32_t row_end = s_win[wi + 1];
            int32_t run_begin = blk_begin;
            Vec<VEC> acc;
            acc.zero();
            // Entries are fetched kDepth at a time regardless of row ends, so
            // that kDepth rows of B are in flight, and then consumed in order;
            // the register is flushed where a row or the block ends.
            for (int32_t p0 = blk_begin; p0 < blk_end; p0 += kDepth) {
                StagedEntry e[kDepth];
                Vec<VEC> b[kDepth];
                if (p0 + kDepth < row_end && p0 + kDepth < blk_end) {
                    // no row or block ends inside this batch: nothing to decide per entry
#pragma unroll
                    for (int u = 0; u < kDepth; ++u) e[u] = s_A[p0 + u - tile_start];
#pragma unroll
                    for (int u = 0; u < kDepth; ++u) b[u] = load_vec<VEC>(Brow.at(e[u].col));
#pragma unroll
                    for (int u = 0; u < kDepth; ++u) acc.fma(e[u].val, b[u]);
                    continue;
                }
#pragma unroll
                for (int u = 0; u < kDepth; ++u) {
                    e[u].col = 0;
                    e[u].val = 0.0f;
                    if (p0 + u < blk_end) e[u] = s_A[p0 + u - tile_start];
                }
#pragma unroll
                for (int u = 0; u < kDepth; ++u) {
                    b[u].zero();
                    if (p0 + u < blk_end) b[u] = load_vec<VEC>(Brow.at(e[u].col));
                }
#pragma unroll
                for (int u = 0; u < kDepth; ++u) {
                    const int32_t p = p0 + u;
                    if (p >= blk_end) continue;
                    acc.fma(e[u].val, b[u]);
                    if (p + 1 != row_end && p + 1 != blk_end) continue;
                    // flush the run [run_begin, p] of the row at window index wi
                    const int32_t row = s_row ? s_row[wi] : row_lb + wi;
                    if constexpr (MERGE) {
                        if (run_begin == row_begin && p + 1 == row_end) {
                            // the run is the whole row
                            store_vec_stream<VEC>(a.C + (int64_t)row * N + k, acc);
                        } else {
                            const int32_t first_in_chunk = row_begin > base ? row_begin : base;
                            const int32_t slot =
                                row_begin < base ? mb.nslots - 1 : (row_begin - tile_start) >> a.log2_group;
                            merge_add<VEC, kCasMerge>(mb, slot, chunk * VEC, acc, chunk == 0 && run_begin == first_in_chunk, row,
                                           row_begin < base || row_end > end);
                        }
                    } else {
                        // the whole row lies inside this aligned block: nobody else adds to it
                        const bool plain = row_begin >= blk && row_end <= blk + G;
                        write_out<LC, VEC>(a, row, k, plain, acc);
                    }
                    acc.zero();
                    if (p + 1 < blk_end) {
                        // next row with stored entries (there is one at or before the
                        // chunk's last row): the very next slot in a window of rows with
                        // entries only, else bisect over the rows without entries
                        ++wi;
                        row_begin = row_end;
                        row_end = s_win[wi + 1];
                        if (row_end <= p + 1) {
                            wi = last_row_at_or_before(s_win, wi + 1, w.n_last, p + 1);
                            row_end = s_win[wi + 1];
                        }
                        run_begin = p + 1;  // = row_begin
                    }
                }
            }
        }
        if constexpr (MERGE) {
            __syncthreads();  // all partial sums of this pass are in LDS
            merge_write_out<LC, VEC>(a, mb, k, k_ok);
            __syncthreads();  // slots are clear again
        }
    }
}

// EPT = tile / kBlock stored entries per thread held in registers between tiles.
template <int LC, int VEC, bool OFF32, bool MERGE, int EPT>
__global__ __launch_bounds__(kBlock) void nnz_serial_kernel(SpmmArgs a)
{
    constexpr int TILE = EPT * kBlock;
    constexpr int WPT = kWindowCap / kBlock + 1;  // rowptr window entries per thread (last one: thread 0 only)
    extern __shared__ __align__(16) unsigned char s_raw[];
    // (the window of rows with entries holds up to one row per position of the tile)
    constexpr int WIN = TILE > kWindowCap ? TILE : kWindowCap;
    __shared__ int32_t s_win[WIN + 1];
    __shared__ int32_t s_row[WIN];
    __shared__ int32_t s_scan[kWavesPerBlock];
    __shared__ int32_t s_tile_row[kTileRowBatch];
    constexpr int WIDTH = LC * VEC;

    StagedEntry* s_A = reinterpret_cast<StagedEntry*>(s_raw);
    MergeBuf mb;
    mb.nslots = TILE / a.group + 1;
    mb.width = WIDTH;
    mb.accum = reinterpret_cast<float*>(s_raw + (size_t)TILE * sizeof(StagedEntry));
    mb.slot_row = reinterpret_cast<int32_t*>(mb.accum + (MERGE ? mb.nslots * WIDTH : 0));
    mb.slot_atomic = mb.slot_row + mb.nslots;

    const int32_t M = (int32_t)a.M;
    const int32_t nnz = a.rowptr[a.M];
    const int64_t tiles = ((int64_t)nnz + TILE - 1) / TILE;
    const TileDeal deal(tiles, blockIdx.x, gridDim.x);
    const int64_t my_tiles = deal.mine;
    if (my_tiles == 0) return;
    const int tid = threadIdx.x;

    if constexpr (MERGE) merge_reset(mb);  // made visible by the barriers below

    // registers that carry the next tile in: its entries and its rowptr window
    int32_t nx_col[EPT];
    float nx_val[EPT];
    int32_t nx_win[WPT];
    auto fetch_tile = [&](int64_t t, int32_t row_lb) {
        const int32_t start = (int32_t)(t * TILE);
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const int32_t p = start + tid + i * kBlock;
            nx_col[i] = 0;
            nx_val[i] = 0.0f;
            if (p < nnz) {
                nx_col[i] = load_stream(a.colidx + p);
                nx_val[i] = load_stream(a.vals + p);
            }
        }
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            const int w = tid + i * kBlock;
            const int64_t r = (int64_t)row_lb + w;
            nx_win[i] = w <= kWindowCap ? a.rowptr[r <= M ? r : M] : 0;
        }
    };

    for (int64_t j0 = 0; j0 < my_tiles; j0 += kTileRowBatch) {
        find_tile_rows(a, deal, j0, TILE, s_tile_row);
        const int64_t j1 = j0 + kTileRowBatch < my_tiles ? j0 + kTileRowBatch : my_tiles;
        fetch_tile(deal.tile(j0), s_tile_row[0]);

        for (int64_t j = j0; j < j1; ++j) {
            const int64_t t = deal.tile(j);
            const int32_t tile_start = (int32_t)(t * TILE);
            const int32_t tile_end = nnz - tile_start < TILE ? nnz : tile_start + TILE;
            int32_t row_lb = s_tile_row[j - j0];

            // install the tile that was fetched ahead
#pragma unroll
            for (int i = 0; i < EPT; ++i) {
                StagedEntry e;
                e.col = nx_col[i];
                e.val = nx_val[i];
                s_A[tid + i * kBlock] = e;
            }
#pragma unroll
            for (int i = 0; i < WPT; ++i)
                if (tid + i * kBlock <= kWindowCap) s_win[tid + i * kBlock] = nx_win[i];
            __syncthreads();
            // start bringing in the next tile of this batch
            if (j + 1 < j1) fetch_tile(deal.tile(j + 1), s_tile_row[j + 1 - j0]);

            // The rows WITH entries of the tile, their first positions in s_win and their numbers in s_row: rows
            // without entries (44 % of the rows of an R-MAT matrix, in runs of 3.5 on average) would cost a search
            // of the window at the end of the row in front of them, and cutting a tile whose rows do not fit the
            // plain window costs a window load and several barriers per cut (R-MAT's sparse end: up to nine cuts
            // per tile).  One path for all tiles also keeps the kernel's code (serial_chunk is long) small.
            RowWindow w;
            w.cnt = tile_end - tile_start;
            w.n_first = 0;
            if (s_win[kWindowCap] >= tile_end) {
                // the plain window covers every row of the tile: cut it down where it stands
                w.n_last = compact_window(s_win, s_row, row_lb, tile_end, s_scan) - 1;
            } else {
                // long runs of rows without entries: read on in rowptr
                __syncthreads();  // everyone has read the plain window
                w.n_last = load_compact_window(a, row_lb, tile_end, s_win, s_row, s_scan) - 1;
            }
            serial_chunk<LC, VEC, OFF32, MERGE>(a, mb, s_A, s_win, w, 0, tile_start, tile_start, tile_end, s_row);
            // tile and window fully consumed before they are overwritten (tile mode ends with a barrier of its own)
            if constexpr (!MERGE) __syncthreads();
        }
    }
}

namespace nnz_serial_detail {

struct Launch {
    const SpmmArgs& a;
    int compute_units;
    int64_t nnz_hint;
    bool off32;
    int tile;
    bool merge;
    hipStream_t s;

    template <int LC, int VEC, bool OFF32, bool MERGE, int EPT>
    void go() const
    {
        const int nslots = tile / a.group + 1;
        const int smem = tile * (int)sizeof(StagedEntry) + (MERGE ? nslots * (LC * VEC * 4 + 8) : 0);
        static int cached[7];  // [log2 group] resident workgroups per CU of this instance, 0 = not asked yet
        int& per_cu = cached[a.log2_group];
        static int asked = 0;  // most dynamic LDS this instance has been allowed so far
        ensure_dynamic_lds(nnz_serial_kernel<LC, VEC, OFF32, MERGE, EPT>, smem, asked);
        if (per_cu == 0) per_cu = resident_per_cu(nnz_serial_kernel<LC, VEC, OFF32, MERGE, EPT>, smem);
        const int grid = persistent_grid(per_cu, compute_units, nnz_hint, tile);
        hipLaunchKernelGGL((nnz_serial_kernel<LC, VEC, OFF32, MERGE, EPT>), dim3(grid), dim3(kBlock), smem, s, a);
    }

    template <int LC, int VEC, bool OFF32, bool MERGE>
    void pick_tile() const
    {
        // the small tiles exist for 16-byte lanes only (plan_nnz_serial)
        if constexpr (VEC == 4) {
            if (tile == 256) return go<LC, VEC, OFF32, MERGE, 1>();
            if (tile == 512) return go<LC, VEC, OFF32, MERGE, 2>();
        }
        if (tile == 1024) go<LC, VEC, OFF32, MERGE, 4>();
        else go<LC, VEC, OFF32, MERGE, 8>();
    }

    template <int LC, int VEC>
    void pick_mode() const
    {
        if (off32) {
            if (merge) pick_tile<LC, VEC, true, true>(); else pick_tile<LC, VEC, true, false>();
        } else {
            if (merge) pick_tile<LC, VEC, false, true>(); else pick_tile<LC, VEC, false, false>();
        }
    }

    // launch the instance for LC chunk lanes per stored entry
    template <int LC>
    hipError_t run(int vec) const
    {
        switch (vec) {
            case 4: pick_mode<LC, 4>(); break;
            case 2: pick_mode<LC, 2>(); break;
            case 1: pick_mode<LC, 1>(); break;
            default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
};

}  // namespace nnz_serial_detail
}  // namespace sgap
