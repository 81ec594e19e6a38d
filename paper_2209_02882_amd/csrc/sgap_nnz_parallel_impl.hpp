// Nnz-balanced schedule, parallel strategy: {<1 nnz, c col>, r} with r = G
// (Section 6.2, the "1 nnz" listing).  The unit of work is a stored entry of A
// (the paper's first atomic-parallelism family, <x nnz, y col>, Section 3.2).
// Stored entries are cut into tiles; a workgroup stages a tile's (column,
// value, row, meta) records in LDS and then lets its lanes combine them.  The
// row of a position is found by searching rowptr, as in the paper's Listings 1
// and 2, but only inside the tile's window of rows, which is kept in LDS.
//
// This header holds the kernel templates and the per-group launcher; it is
// included by the sgap_nnz_parallel_g*.hip translation units, each of which
// instantiates the kernels of a few group sizes (the instances are split over
// several files only to compile them side by side).
#pragma once
#include "sgap_common.hpp"
#include "sgap_lane_ops.hpp"
#include "sgap_nnz_common.hpp"

namespace sgap {

// LDS record of one stored entry
struct __align__(16) TileEntry {
    int32_t col;
    float val;
    int32_t row;
    int32_t meta;
};
constexpr int kMetaLeftMask = 127;       // min(entries left in the row after this one, 127): more than any group
constexpr int kMetaValid = 1 << 7;       // position inside the chunk
constexpr int kMetaRowStart = 1 << 8;    // first stored entry of its row
constexpr int kMetaChunkStart = 1 << 9;  // first position of the chunk (a run starts here too)
constexpr int kMetaOwner = 1 << 10;      // first entry of its row inside the chunk
constexpr int kMetaOutside = 1 << 11;    // the row also has entries outside the chunk
constexpr int kMetaPlain = 1 << 12;      // direct mode: row lies inside one aligned block of `group`
constexpr int kMetaSlotShift = 16;       // tile mode: LDS accumulator slot of the row

constexpr int kParEpt = kParTile / kBlock;     // stored entries per thread held in registers between tiles
constexpr int kParWpt = kWindowCap / kBlock + 1;
// LDS merge through the hardware's fp32 atomic: the run heads of one row meet on
// one address within a wavefront (measured against the compare-and-swap loop:
// rmat N=4 G=16 0.47 vs 0.62 ms, powerlaw 0.135 vs 0.162 ms)
constexpr bool kParMergeCas = false;
constexpr int kParDepth = 4;                   // steps issued together

// Build the LDS records of the chunk [base, end) of the tile that starts at
// tile_start from the entries a thread holds in registers (thread t holds
// positions tile_start + t + i*kBlock).  LDS slot s holds position
// tile_start + s; slots outside the chunk are marked invalid.  The rows of the
// chunk are s_win[w.n_first .. w.n_last + 1] relative to row_lb, or, when s_row is
// given (a window of the rows with entries only), the rows s_row[wi]; s_row may
// then lie inside s_tile: every thread has read its rows before any record is
// written (a barrier in between, so the call is block-uniform in that case).
__device__ __forceinline__ void build_records(const int32_t (&col)[kParEpt], const float (&val)[kParEpt],
                                              int32_t tile_start, int32_t base, int32_t end, const RowWindow& w,
                                              int32_t row_lb, int log2_group, int nslots,
                                              const int32_t* __restrict__ s_win, TileEntry* s_tile,
                                              const int32_t* s_row = nullptr)
{
    TileEntry rec[kParEpt];
#pragma unroll
    for (int i = 0; i < kParEpt; ++i) {
        const int q = threadIdx.x + i * kBlock;
        const int32_t p = tile_start + q;
        TileEntry e;
        e.col = 0; e.val = 0.0f; e.row = 0; e.meta = 0;
        if (p >= base && p < end) {
            const int32_t wi = last_row_at_or_before(s_win, w.n_first, w.n_last, p);
            const int32_t p_begin = s_win[wi];
            const int32_t p_end = s_win[wi + 1];
            const int32_t left = p_end - 1 - p;
            int32_t meta = kMetaValid | (left < kMetaLeftMask ? left : kMetaLeftMask);
            if (p == p_begin) meta |= kMetaRowStart;
            if (p == base) meta |= kMetaChunkStart;
            if (p == (p_begin > base ? p_begin : base)) meta |= kMetaOwner;
            if (p_begin < base || p_end > end) meta |= kMetaOutside;
            if ((p_begin >> log2_group) == ((p_end - 1) >> log2_group)) meta |= kMetaPlain;
            const int32_t slot = p_begin < base ? nslots - 1 : (p_begin - tile_start) >> log2_group;
            meta |= slot << kMetaSlotShift;
            e.col = col[i];
            e.val = val[i];
            e.row = s_row ? s_row[wi] : row_lb + wi;
            e.meta = meta;
        }
        rec[i] = e;
    }
    if (s_row) __syncthreads();
#pragma unroll
    for (int i = 0; i < kParEpt; ++i) s_tile[threadIdx.x + i * kBlock] = rec[i];
}

// Multiply out the records staged in s_tile: a lane multiplies ONE stored
// entry by its column chunk; the G members of a group then run a segmented
// sum keyed by row and the first lane of every run writes.  Lanes outside the
// chunk contribute +0.  Ends with a barrier.
template <int G, int LC, int VEC, bool OFF32, bool MERGE>
__device__ __forceinline__ void parallel_chunk(const SpmmArgs& a, const MergeBuf& mb,
                                               const TileEntry* __restrict__ s_tile)
{
    constexpr int ENTRIES_PER_WAVE = kWave / LC;  // positions one wave covers per step
    constexpr int ENTRIES_PER_STEP = ENTRIES_PER_WAVE * kWavesPerBlock;
    constexpr int STEPS = kParTile / ENTRIES_PER_STEP;
    static_assert(STEPS % kParDepth == 0, "steps are issued kParDepth at a time");
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int entry_lane = lane / LC;  // = slot*G + member
    const int member = entry_lane % G;
    const int chunk = lane % LC;
    const int64_t N = a.N;

    for (int64_t k0 = 0; k0 < N; k0 += (int64_t)LC * VEC) {
        const int64_t k = k0 + (int64_t)chunk * VEC;
        const bool k_ok = k < N;
        const BRow<OFF32> Brow(a.B, N, k);
        for (int step = 0; step < STEPS; step += kParDepth) {
            TileEntry e[kParDepth];
            Vec<VEC> x[kParDepth];
#pragma unroll
            for (int u = 0; u < kParDepth; ++u)
                e[u] = s_tile[((step + u) * kWavesPerBlock + wave) * ENTRIES_PER_WAVE + entry_lane];
#pragma unroll
            for (int u = 0; u < kParDepth; ++u) {
                x[u].zero();
                if ((e[u].meta & kMetaValid) && k_ok) x[u] = load_vec<VEC>(Brow.at(e[u].col));
            }
#pragma unroll
            for (int u = 0; u < kParDepth; ++u) {
                const int32_t meta = e[u].meta;
                const bool valid = (meta & kMetaValid) != 0;
                const int left = meta & kMetaLeftMask;
                const int span = left < G - 1 - member ? left : G - 1 - member;
#pragma unroll
                for (int i = 0; i < VEC; ++i) x[u].v[i] = group_seg_sum<G, LC>(e[u].val * x[u].v[i], span);
                // a run starts at member 0, at a row's first entry and at the chunk's first position
                const bool head = valid && (member == 0 || (meta & (kMetaRowStart | kMetaChunkStart)));
                if (head && k_ok) {
                    if constexpr (MERGE) {
                        if ((meta & kMetaRowStart) && left <= G - 1 - member) {
                            // the run is the whole row
                            store_vec_stream<VEC>(a.C + (int64_t)e[u].row * N + k, x[u]);
                        } else {
                            merge_add<VEC, kParMergeCas>(mb, meta >> kMetaSlotShift, chunk * VEC, x[u],
                                           chunk == 0 && (meta & kMetaOwner), e[u].row, (meta & kMetaOutside) != 0);
                        }
                    } else {
                        write_out<LC, VEC>(a, e[u].row, k, (meta & kMetaPlain) != 0, x[u]);
                    }
                }
            }
        }
        if constexpr (MERGE) {
            __syncthreads();  // all partial sums of this pass are in LDS
            merge_write_out<LC, VEC>(a, mb, k, k_ok);
        }
        __syncthreads();  // slots clear / records fully consumed
    }
}

// {<1 nnz, c col>, r} with r = G (Section 6.2, the "1 nnz" listing; Listing 2
// is its G = 32 instance).
//   lane = (slot*G + member)*LC + chunk ; member <-> consecutive positions
// Tiles are handed out by TileDeal; the loads that bring in the next tile (entries
// and rowptr window) are issued before the current tile is multiplied out.
// MERGE selects tile mode of the merge rule.
template <int G, int LC, int VEC, bool OFF32, bool MERGE>
__global__ __launch_bounds__(kBlock) void nnz_parallel_kernel(SpmmArgs a)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    __shared__ int32_t s_win[kWindowCap + 1];
    __shared__ int32_t s_scan[kWavesPerBlock];
    __shared__ int32_t s_tile_row[kTileRowBatch];
    constexpr int WIDTH = LC * VEC;
    static_assert(kParTile <= kWindowCap, "the window of rows with entries holds one row per position");
    static_assert(kWindowCap * sizeof(int32_t) <= kParTile * sizeof(TileEntry), "those rows are staged in the record area");

    TileEntry* s_tile = reinterpret_cast<TileEntry*>(s_raw);
    MergeBuf mb;
    mb.nslots = kParTile / G + 1;
    mb.width = WIDTH;
    mb.accum = reinterpret_cast<float*>(s_raw + (size_t)kParTile * sizeof(TileEntry));
    mb.slot_row = reinterpret_cast<int32_t*>(mb.accum + (MERGE ? mb.nslots * WIDTH : 0));
    mb.slot_atomic = mb.slot_row + mb.nslots;

    const int32_t M = (int32_t)a.M;
    const int32_t nnz = a.rowptr[a.M];
    const int64_t tiles = ((int64_t)nnz + kParTile - 1) / kParTile;
    const TileDeal deal(tiles, blockIdx.x, gridDim.x);
    const int64_t my_tiles = deal.mine;
    if (my_tiles == 0) return;
    const int tid = threadIdx.x;

    if constexpr (MERGE) merge_reset(mb);  // made visible by the barriers below

    // registers that carry a tile in: its entries and its rowptr window
    int32_t nx_col[kParEpt];
    float nx_val[kParEpt];
    int32_t nx_win[kParWpt];
    auto fetch_tile = [&](int64_t t, int32_t row_lb) {
        const int32_t start = (int32_t)(t * kParTile);
#pragma unroll
        for (int i = 0; i < kParEpt; ++i) {
            const int32_t p = start + tid + i * kBlock;
            nx_col[i] = 0;
            nx_val[i] = 0.0f;
            if (p < nnz) {
                nx_col[i] = load_stream(a.colidx + p);
                nx_val[i] = load_stream(a.vals + p);
            }
        }
#pragma unroll
        for (int i = 0; i < kParWpt; ++i) {
            const int w = tid + i * kBlock;
            const int64_t r = (int64_t)row_lb + w;
            nx_win[i] = w <= kWindowCap ? a.rowptr[r <= M ? r : M] : 0;
        }
    };

    for (int64_t j0 = 0; j0 < my_tiles; j0 += kTileRowBatch) {
        find_tile_rows(a, deal, j0, kParTile, s_tile_row);
        const int64_t j1 = j0 + kTileRowBatch < my_tiles ? j0 + kTileRowBatch : my_tiles;
        fetch_tile(deal.tile(j0), s_tile_row[0]);

        for (int64_t j = j0; j < j1; ++j) {
            const int64_t t = deal.tile(j);
            const int32_t tile_start = (int32_t)(t * kParTile);
            const int32_t tile_end = nnz - tile_start < kParTile ? nnz : tile_start + kParTile;
            int32_t row_lb = s_tile_row[j - j0];

            // install the window that was fetched ahead
#pragma unroll
            for (int i = 0; i < kParWpt; ++i)
                if (tid + i * kBlock <= kWindowCap) s_win[tid + i * kBlock] = nx_win[i];
            __syncthreads();

            if (s_win[kWindowCap] >= tile_end) {
                // the window covers every row of the tile: one chunk
                RowWindow w;
                w.cnt = tile_end - tile_start;
                w.n_first = first_above(s_win, kWindowCap + 1, tile_start) - 1;
                w.n_last = first_above(s_win, kWindowCap + 1, tile_end - 1) - 1;
                build_records(nx_col, nx_val, tile_start, tile_start, tile_end, w, row_lb, a.log2_group, mb.nslots,
                              s_win, s_tile);
                __syncthreads();
                // start bringing in the next tile of this batch
                if (j + 1 < j1) fetch_tile(deal.tile(j + 1), s_tile_row[j + 1 - j0]);
                parallel_chunk<G, LC, VEC, OFF32, MERGE>(a, mb, s_tile);
            } else {
                // long runs of rows without entries: a window of the rows with entries only, so that the tile
                // still goes in one piece (sgap_nnz_common.hpp).  The rows are staged in the record area, which is
                // free until build_records fills it (no static LDS to spare beside the largest merge slots).
                int32_t* s_row = reinterpret_cast<int32_t*>(s_tile);
                __syncthreads();  // everyone has read the plain window
                RowWindow w;
                w.cnt = tile_end - tile_start;
                w.n_first = 0;
                w.n_last = load_compact_window(a, row_lb, tile_end, s_win, s_row, s_scan) - 1;
                build_records(nx_col, nx_val, tile_start, tile_start, tile_end, w, 0, a.log2_group, mb.nslots, s_win,
                              s_tile, s_row);
                __syncthreads();
                if (j + 1 < j1) fetch_tile(deal.tile(j + 1), s_tile_row[j + 1 - j0]);
                parallel_chunk<G, LC, VEC, OFF32, MERGE>(a, mb, s_tile);
            }
        }
    }
}

namespace nnz_parallel_detail {

struct Launch {
    const SpmmArgs& a;
    int compute_units;
    int64_t nnz_hint;
    bool off32;
    bool merge;
    hipStream_t s;

    template <int G, int LC, int VEC, bool OFF32, bool MERGE>
    void go() const
    {
        constexpr int nslots = kParTile / G + 1;
        constexpr int smem = kParTile * (int)sizeof(TileEntry) + (MERGE ? nslots * (LC * VEC * 4 + 8) : 0);
        static int asked = 0;
        ensure_dynamic_lds(nnz_parallel_kernel<G, LC, VEC, OFF32, MERGE>, smem, asked);
        static const int per_cu = resident_per_cu(nnz_parallel_kernel<G, LC, VEC, OFF32, MERGE>, smem);
        const int grid = persistent_grid(per_cu, compute_units, nnz_hint, kParTile);
        hipLaunchKernelGGL((nnz_parallel_kernel<G, LC, VEC, OFF32, MERGE>), dim3(grid), dim3(kBlock), smem, s, a);
    }

    template <int G, int LC, int VEC>
    void operator()() const
    {
        if (off32) {
            if (merge) go<G, LC, VEC, true, true>(); else go<G, LC, VEC, true, false>();
        } else {
            if (merge) go<G, LC, VEC, false, true>(); else go<G, LC, VEC, false, false>();
        }
    }
};

// launch the instance for group size G (lc * G <= 64)
template <int G>
inline hipError_t launch_group(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, bool merge,
                               hipStream_t s)
{
    if (!dispatch_lc<G>(lc, vec, Launch{a, compute_units, nnz_hint, offsets_fit_32(a), merge, s}))
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace nnz_parallel_detail
}  // namespace sgap
