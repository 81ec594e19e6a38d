// Nnz-balanced schedule, parallel strategy, and the row-zeroing pass of the
// schedule.  The unit of work is a stored entry of A (the paper's first
// atomic-parallelism family, <x nnz, y col>, Section 3.2).  Stored entries are
// cut into chunks; a workgroup stages a chunk's (column, value, row, meta)
// records in LDS and then lets its lanes combine them.  The row of a position
// is found by searching rowptr, as in the paper's Listings 1 and 2, but only
// inside the chunk's window of rows, which is kept in LDS.
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

// Stage the chunk of positions starting at `base` (up to the tile's end, or as
// many as the row window covers, see load_row_window) into LDS and return how
// many positions were staged.  LDS slot s holds position tile_start + s; slots
// outside the chunk are marked invalid.  `row_lb` is any row with rowptr[row_lb] <= base; on return
// it is the row of the chunk's last position (a valid lower bound for the
// next chunk).  Block-uniform control flow; ends with a barrier.
__device__ __forceinline__ int32_t stage_tile(const SpmmArgs& a, int32_t base, int32_t tile_start, int32_t tile_end,
                                              int tile, int log2_group, int nslots, TileEntry* __restrict__ s_tile,
                                              int32_t* __restrict__ s_win, int32_t& row_lb)
{
    const int tid = threadIdx.x;
    const RowWindow w = load_row_window(a, row_lb, base, tile_end - base, s_win);
    const int32_t end = base + w.cnt;

    for (int q = tid; q < tile; q += kBlock) {
        TileEntry e;
        e.col = 0; e.val = 0.0f; e.row = 0; e.meta = 0;
        const int32_t p = tile_start + q;
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
            e.col = load_stream(a.colidx + p);
            e.val = load_stream(a.vals + p);
            e.row = row_lb + wi;
            e.meta = meta;
        }
        s_tile[q] = e;
    }
    row_lb += w.n_last;
    __syncthreads();
    return w.cnt;
}

// {<1 nnz, c col>, r} with r = G (Section 6.2, the "1 nnz" listing; Listing 2
// is its G = 32 instance): a lane multiplies ONE stored entry by its column
// chunk; the G members of a group then run a segmented sum keyed by row and
// the first lane of every run writes.  Lanes outside the chunk contribute +0.
//   lane = (slot*G + member)*LC + chunk ; member <-> consecutive positions
// kParDepth steps are issued together so that several gathered rows of B are
// in flight per lane.  MERGE selects tile mode of the merge rule.
constexpr int kParDepth = 4;

template <int G, int LC, int VEC, bool OFF32, bool MERGE>
__global__ __launch_bounds__(kBlock) void nnz_parallel_kernel(SpmmArgs a, int tile)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    __shared__ int32_t s_win[kWindowCap + 1];
    constexpr int ENTRIES_PER_WAVE = kWave / LC;  // positions one wave covers per step
    constexpr int ENTRIES_PER_STEP = ENTRIES_PER_WAVE * kWavesPerBlock;
    constexpr int WIDTH = LC * VEC;

    TileEntry* s_tile = reinterpret_cast<TileEntry*>(s_raw);
    MergeBuf mb;
    mb.nslots = tile / G + 1;
    mb.width = WIDTH;
    mb.accum = reinterpret_cast<float*>(s_raw + (size_t)tile * sizeof(TileEntry));
    mb.slot_row = reinterpret_cast<int32_t*>(mb.accum + (MERGE ? mb.nslots * WIDTH : 0));
    mb.slot_atomic = mb.slot_row + mb.nslots;

    const int32_t nnz = a.rowptr[a.M];
    const int64_t tiles = ((int64_t)nnz + tile - 1) / tile;
    if ((int64_t)blockIdx.x >= tiles) return;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int entry_lane = lane / LC;  // = slot*G + member
    const int member = entry_lane % G;
    const int chunk = lane % LC;
    const int64_t N = a.N;
    const int steps = tile / ENTRIES_PER_STEP;  // host keeps this a multiple of kParDepth

    if constexpr (MERGE) merge_reset(mb);  // made visible by the first chunk's barriers

    int32_t row_lb = 0;
    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
      const int32_t tile_start = (int32_t)(t * tile);
      const int32_t tile_end = nnz - tile_start < tile ? nnz : tile_start + tile;
      row_lb = find_row_cooperative(a.rowptr, row_lb, (int32_t)a.M - 1, tile_start);
      // a tile is normally one chunk; see load_row_window for when it is cut
      for (int32_t base = tile_start; base < tile_end;) {
        base += stage_tile(a, base, tile_start, tile_end, tile, a.log2_group, mb.nslots, s_tile, s_win, row_lb);
        for (int64_t k0 = 0; k0 < N; k0 += (int64_t)LC * VEC) {
            const int64_t k = k0 + (int64_t)chunk * VEC;
            const bool k_ok = k < N;
            const BRow<OFF32> Brow(a.B, N, k);
            for (int step = 0; step < steps; step += kParDepth) {
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
                                merge_add<VEC>(mb, meta >> kMetaSlotShift, chunk * VEC, x[u],
                                               chunk == 0 && (meta & kMetaOwner), e[u].row, (meta & kMetaOutside) != 0);
                            }
                        } else {
                            write_out<VEC>(a, e[u].row, k, (meta & kMetaPlain) != 0, x[u]);
                        }
                    }
                }
            }
            if constexpr (MERGE) {
                __syncthreads();  // all partial sums of this pass are in LDS
                merge_write_out<LC, VEC>(a, mb, k, k_ok);
            }
            __syncthreads();  // slots clear / tile fully consumed
        }
      }
    }
}

// Rows that will receive global atomic adds (their positions straddle an
// aligned merge block of 2^merge_log2 positions) and rows without stored
// entries are set to +0.
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
    const bool plain = p_end > p_begin && (p_begin >> merge_log2) == ((p_end - 1) >> merge_log2);
    if (plain) return;
    Vec<VEC> z;
    z.zero();
    float* __restrict__ dst = a.C + row * a.N;
    for (int64_t k = (int64_t)chunk * VEC; k < a.N; k += (int64_t)lcz * VEC) store_vec<VEC>(dst + k, z);
}

namespace {

constexpr int kMergeLdsBudget = 34 * 1024;  // bytes of LDS accumulators tile mode may take

struct LaunchNnzParallel {
    const SpmmArgs& a;
    int compute_units;
    int64_t nnz_hint;
    bool off32;
    int tile;
    bool merge;
    hipStream_t s;

    template <int G, int LC, int VEC, bool OFF32, bool MERGE>
    void go() const
    {
        const int nslots = tile / G + 1;
        const int smem = tile * (int)sizeof(TileEntry) + (MERGE ? nslots * (LC * VEC * 4 + 8) : 0);
        static const int per_cu = resident_per_cu(nnz_parallel_kernel<G, LC, VEC, OFF32, MERGE>, smem);
        const int grid = persistent_grid(per_cu, compute_units, nnz_hint, tile);
        hipLaunchKernelGGL((nnz_parallel_kernel<G, LC, VEC, OFF32, MERGE>), dim3(grid), dim3(kBlock), smem, s, a,
                           tile);
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
}  // namespace

NnzPlan plan_nnz_parallel(int group, int lc, int vec)
{
    NnzPlan p;
    // one step covers 4*64/lc positions; kParDepth steps per batch; at least 1024
    const int per_batch = (kWave / lc) * kWavesPerBlock * kParDepth;
    p.tile = per_batch > 1024 ? per_batch : 1024;
    const int nslots = p.tile / group + 1;
    p.merge = nslots * (lc * vec * 4 + 8) <= kMergeLdsBudget;
    int lg = 0;
    while ((1 << lg) < (p.merge ? p.tile : group)) ++lg;
    p.merge_log2 = lg;
    return p;
}

hipError_t launch_nnz_parallel(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, hipStream_t s)
{
    const NnzPlan plan = plan_nnz_parallel(a.group, lc, vec);
    if (!dispatch_group(a.group, lc, vec,
                        LaunchNnzParallel{a, compute_units, nnz_hint, offsets_fit_32(a), plan.tile, plan.merge, s}))
        return hipErrorInvalidValue;
    return hipGetLastError();
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
