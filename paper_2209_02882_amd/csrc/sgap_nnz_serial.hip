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
// entries need no per-entry row record.
#include "sgap_common.hpp"
#include "sgap_gather.hpp"
#include "sgap_nnz_common.hpp"

namespace sgap {

constexpr int kDepth = 8;  // gathered rows of B in flight per lane

template <int LC, int VEC, bool OFF32>
__global__ __launch_bounds__(kBlock) void nnz_serial_kernel(SpmmArgs a, int tile)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    StagedEntry* s_A = reinterpret_cast<StagedEntry*>(s_raw);
    __shared__ int32_t s_win[kWindowCap + 1];
    constexpr int ENTRY_LANES = kBlock / LC;

    const int32_t nnz = a.rowptr[a.M];
    const PosRange pr = my_positions(nnz, tile);
    if (pr.begin >= pr.end) return;

    const int entry_lane = threadIdx.x / LC;
    const int chunk = threadIdx.x % LC;
    const int64_t N = a.N;
    const int G = a.group;
    const int per_step = ENTRY_LANES * G;  // positions the workgroup covers per step

    const int32_t g_mask = G - 1;
    int32_t row_lb = last_row_at_or_before(a.rowptr, 0, (int32_t)a.M - 1, (int32_t)pr.begin);
    for (int32_t base = (int32_t)pr.begin; base < (int32_t)pr.end;) {
        // LDS slot s holds position slot0 + s, where slot0 is `base` rounded
        // down to a multiple of G: lanes always own globally aligned blocks
        const int32_t slot0 = base & ~g_mask;
        const int32_t room = tile - (base - slot0);
        const int32_t want = (int32_t)pr.end - base < room ? (int32_t)pr.end - base : room;
        const RowWindow w = load_row_window(a, row_lb, base, want, s_win);
        const int32_t end = base + w.cnt;
        stage_entries(a, (uint32_t)base, (uint32_t)w.cnt, s_A + (base - slot0));
        __syncthreads();

        for (int64_t k0 = 0; k0 < N; k0 += (int64_t)LC * VEC) {
            const int64_t k = k0 + (int64_t)chunk * VEC;
            if (k >= N) continue;
            const BRow<OFF32> Brow(a.B, N, k);
            for (int32_t blk = slot0 + entry_lane * G; blk < end; blk += per_step) {
                // this lane's aligned block of G positions, clipped to the chunk
                const int32_t blk_begin = blk > base ? blk : base;
                const int32_t blk_end = blk + G < end ? blk + G : end;
                if (blk_begin >= blk_end) continue;
                // window index of the row that holds blk_begin
                int32_t wi = last_row_at_or_before(s_win, w.n_first, w.n_last, blk_begin);
                int32_t row_begin = s_win[wi];
                int32_t row_end = s_win[wi + 1];
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
                        if (p0 + u < blk_end) e[u] = s_A[p0 + u - slot0];
                    }
#pragma unroll
                    for (int u = 0; u < kDepth; ++u) {
                        b[u].zero();
                        if (p0 + u < blk_end) b[u] = load_vec<VEC>(Brow.at(e[u].col));
                    }
#pragma unroll
                    for (int u = 0; u < kDepth; ++u) {
                        const int32_t p = p0 + u;
                        if (p < blk_end) {
                            acc.fma(e[u].val, b[u]);
                            if (p + 1 == row_end || p + 1 == blk_end) {
                                // the whole row lies inside this aligned block: nobody else adds to it
                                const bool plain = row_begin >= blk && row_end <= blk + G;
                                write_out<VEC>(a, row_lb + wi, k, plain, acc);
                                acc.zero();
                                if (p + 1 < blk_end) {
                                    // next row with stored entries (there is one at or
                                    // before the chunk's last row): usually the very
                                    // next row, else bisect over the rows without entries
                                    ++wi;
                                    row_begin = row_end;
                                    row_end = s_win[wi + 1];
                                    if (row_end <= p + 1) {
                                        wi = last_row_at_or_before(s_win, wi + 1, w.n_last, p + 1);
                                        row_end = s_win[wi + 1];
                                    }
                                }
                            }
                        }
                    }
                }
            }
        }
        row_lb += w.n_last;
        base = end;
        __syncthreads();  // chunk and window fully consumed before they are overwritten
    }
}

namespace {
struct LaunchNnzSerial {
    const SpmmArgs& a;
    int compute_units;
    int64_t nnz_hint;
    bool off32;
    hipStream_t s;
    template <int G, int LC, int VEC>
    void operator()() const
    {
        // keep every entry lane busy: tile >= lanes * group, within 1024..4096 positions
        int tile = 1024;
        while (tile < 4096 && tile < (kBlock / LC) * a.group) tile *= 2;
        const int smem = tile * (int)sizeof(StagedEntry);
        static int cached[2][3] = {{0, 0, 0}, {0, 0, 0}};  // [off32][tile] resident workgroups per CU
        int& per_cu = cached[off32 ? 1 : 0][tile == 1024 ? 0 : tile == 2048 ? 1 : 2];
        if (per_cu == 0)
            per_cu = off32 ? resident_per_cu(nnz_serial_kernel<LC, VEC, true>, smem)
                           : resident_per_cu(nnz_serial_kernel<LC, VEC, false>, smem);
        const int grid = persistent_grid(per_cu, compute_units, nnz_hint, tile);
        if (off32)
            hipLaunchKernelGGL((nnz_serial_kernel<LC, VEC, true>), dim3(grid), dim3(kBlock), smem, s, a, tile);
        else
            hipLaunchKernelGGL((nnz_serial_kernel<LC, VEC, false>), dim3(grid), dim3(kBlock), smem, s, a, tile);
    }
};
}  // namespace

hipError_t launch_nnz_serial(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, hipStream_t s)
{
    // group is a run-time count here; dispatch on (lc, vec) only
    if (!dispatch_lc<1>(lc, vec, LaunchNnzSerial{a, compute_units, nnz_hint, offsets_fit_32(a), s}))
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace sgap
