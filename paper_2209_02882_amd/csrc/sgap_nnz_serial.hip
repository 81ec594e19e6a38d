// Nnz-balanced schedule, serial strategy: {<g nnz, c col>, 1} (Section 6.1,
// the "g nnz" listing).  The unit of work is a stored entry of A; a lane walks
// `group` consecutive stored entries by itself and flushes its register
// whenever the row ends or its share ends (conditional reduction).
//   thread = entry_lane*LC + chunk over the whole workgroup
//
// A workgroup copies a chunk of (column, value) pairs into LDS together with
// the window of rowptr the chunk touches.  A lane finds the row of its first
// position by searching that window (Listings 1 and 2 search rowptr the same
// way) and then follows the row ends through the window, so the stored
// entries need no per-entry row record.
#include "sgap_common.hpp"
#include "sgap_gather.hpp"
#include "sgap_nnz_common.hpp"

namespace sgap {

constexpr int kDepth = 8;  // gathered rows of B in flight per lane

// MERGE selects tile mode of the merge rule (see sgap_nnz_common.hpp).
template <int LC, int VEC, bool OFF32, bool MERGE>
__global__ __launch_bounds__(kBlock) void nnz_serial_kernel(SpmmArgs a, int tile)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    __shared__ int32_t s_win[kWindowCap + 1];
    constexpr int ENTRY_LANES = kBlock / LC;
    constexpr int WIDTH = LC * VEC;

    const int G = a.group;
    StagedEntry* s_A = reinterpret_cast<StagedEntry*>(s_raw);
    MergeBuf mb;
    mb.nslots = tile / G + 1;
    mb.width = WIDTH;
    mb.accum = reinterpret_cast<float*>(s_raw + (size_t)tile * sizeof(StagedEntry));
    mb.slot_row = reinterpret_cast<int32_t*>(mb.accum + (MERGE ? mb.nslots * WIDTH : 0));
    mb.slot_atomic = mb.slot_row + mb.nslots;

    const int32_t nnz = a.rowptr[a.M];
    const int64_t tiles = ((int64_t)nnz + tile - 1) / tile;
    if ((int64_t)blockIdx.x >= tiles) return;

    const int entry_lane = threadIdx.x / LC;
    const int chunk = threadIdx.x % LC;
    const int64_t N = a.N;
    const int per_step = ENTRY_LANES * G;  // positions the workgroup covers per step

    if constexpr (MERGE) merge_reset(mb);  // made visible by the first chunk's barriers

    int32_t row_lb = 0;
    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
      const int32_t tile_start = (int32_t)(t * tile);
      const int32_t tile_end = nnz - tile_start < tile ? nnz : tile_start + tile;
      row_lb = find_row_cooperative(a.rowptr, row_lb, (int32_t)a.M - 1, tile_start);
      // A tile is normally one chunk; it is cut into several (at row
      // boundaries) only where its rows do not fit the LDS window.  LDS slot s
      // holds position tile_start + s, so lanes own globally aligned blocks.
      for (int32_t base = tile_start; base < tile_end;) {
        const RowWindow w = load_row_window(a, row_lb, base, tile_end - base, s_win);
        const int32_t end = base + w.cnt;
        stage_entries(a, (uint32_t)base, (uint32_t)w.cnt, s_A + (base - tile_start));
        __syncthreads();

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
                // Entries are fetched kDepth at a time regardless of row ends,
                // so that kDepth rows of B are in flight, and then consumed in
                // order; the register is flushed where a row or the block ends.
                for (int32_t p0 = blk_begin; p0 < blk_end; p0 += kDepth) {
                    StagedEntry e[kDepth];
                    Vec<VEC> b[kDepth];
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
                        // flush the run [run_begin, p] of row row_lb + wi
                        const int32_t row = row_lb + wi;
                        if constexpr (MERGE) {
                            if (run_begin == row_begin && p + 1 == row_end) {
                                // the run is the whole row
                                store_vec_stream<VEC>(a.C + (int64_t)row * N + k, acc);
                            } else {
                                const int32_t first_in_chunk = row_begin > base ? row_begin : base;
                                const int32_t slot = row_begin < base ? mb.nslots - 1 : (row_begin - tile_start) >> a.log2_group;
                                merge_add<VEC>(mb, slot, chunk * VEC, acc, chunk == 0 && run_begin == first_in_chunk,
                                               row, row_begin < base || row_end > end);
                            }
                        } else {
                            // the whole row lies inside this aligned block: nobody else adds to it
                            const bool plain = row_begin >= blk && row_end <= blk + G;
                            write_out<VEC>(a, row, k, plain, acc);
                        }
                        acc.zero();
                        if (p + 1 < blk_end) {
                            // next row with stored entries (there is one at or before
                            // the chunk's last row): usually the very next row, else
                            // bisect over the rows without entries
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
        row_lb += w.n_last;
        base = end;
        __syncthreads();  // chunk and window fully consumed before they are overwritten
      }
    }
}

namespace {

constexpr int kMergeLdsBudget = 34 * 1024;  // bytes of LDS accumulators tile mode may take

struct LaunchNnzSerial {
    const SpmmArgs& a;
    int compute_units;
    int64_t nnz_hint;
    bool off32;
    int tile;
    bool merge;
    hipStream_t s;

    template <int LC, int VEC, bool OFF32, bool MERGE>
    void go() const
    {
        const int nslots = tile / a.group + 1;
        const int smem = tile * (int)sizeof(StagedEntry) + (MERGE ? nslots * (LC * VEC * 4 + 8) : 0);
        static int cached[7][3];  // [log2 group][tile class] resident workgroups per CU, 0 = not asked yet
        int& per_cu = cached[a.log2_group][tile == 1024 ? 0 : tile == 2048 ? 1 : 2];
        if (per_cu == 0) per_cu = resident_per_cu(nnz_serial_kernel<LC, VEC, OFF32, MERGE>, smem);
        const int grid = persistent_grid(per_cu, compute_units, nnz_hint, tile);
        hipLaunchKernelGGL((nnz_serial_kernel<LC, VEC, OFF32, MERGE>), dim3(grid), dim3(kBlock), smem, s, a, tile);
    }

    template <int G, int LC, int VEC>
    void operator()() const
    {
        if (off32) {
            if (merge) go<LC, VEC, true, true>(); else go<LC, VEC, true, false>();
        } else {
            if (merge) go<LC, VEC, false, true>(); else go<LC, VEC, false, false>();
        }
    }
};
}  // namespace

// Tile size and merge mode of the serial kernel for a given layout; the
// zeroing pass must be launched with the same merge_log2.
NnzPlan plan_nnz_serial(int group, int lc, int vec)
{
    NnzPlan p;
    // keep every entry lane busy: tile >= lanes * group, within 1024..4096 positions
    p.tile = 1024;
    while (p.tile < 4096 && p.tile < (kBlock / lc) * group) p.tile *= 2;
    const int nslots = p.tile / group + 1;
    p.merge = nslots * (lc * vec * 4 + 8) <= kMergeLdsBudget;
    int lg = 0;
    while ((1 << lg) < (p.merge ? p.tile : group)) ++lg;
    p.merge_log2 = lg;
    return p;
}

hipError_t launch_nnz_serial(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, hipStream_t s)
{
    const NnzPlan plan = plan_nnz_serial(a.group, lc, vec);
    // group is a run-time count here; dispatch on (lc, vec) only
    if (!dispatch_lc<1>(lc, vec,
                        LaunchNnzSerial{a, compute_units, nnz_hint, offsets_fit_32(a), plan.tile, plan.merge, s}))
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace sgap
