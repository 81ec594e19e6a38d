// Nnz-balanced schedule, parallel strategy, and the row-zeroing pass of the
// schedule.  The unit of work is a stored entry of A (the paper's first
// atomic-parallelism family, <x nnz, y col>, Section 3.2).  Stored entries are
// cut into tiles; a workgroup stages a tile's (column, value, row, meta)
// records in LDS and then lets its lanes combine them.  The row of a position
// is found by searching rowptr, as in the paper's Listings 1 and 2, but only
// inside the tile's window of rows, which is kept in LDS when it fits.
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
constexpr int kMetaSpanMask = 63;      // min(entries left in the row after this one, 63)
constexpr int kMetaRowStart = 1 << 8;  // first stored entry of its row
constexpr int kMetaPlain = 1 << 9;     // row lies inside one aligned block of `group` positions
constexpr int kMetaValid = 1 << 10;    // position < nnz

// Stage the chunk of positions starting at `base` (as many as fit the tile and
// the row window, see load_row_window) into LDS and return how many positions
// were staged.  LDS slot s holds position slot0 + s, where slot0 is `base`
// rounded down to a multiple of `group`, so that the lanes of a group always
// own a globally aligned block of positions; slots outside the chunk are
// marked invalid.  `row_lb` is any row with rowptr[row_lb] <= base; on return
// it is the row of the chunk's last position (a valid lower bound for the
// next chunk).  Block-uniform control flow; ends with a barrier.
__device__ __forceinline__ int32_t stage_tile(const SpmmArgs& a, int32_t base, int32_t range_end, int tile,
                                              int group, int log2_group, TileEntry* __restrict__ s_tile,
                                              int32_t* __restrict__ s_win, int32_t& row_lb)
{
    const int tid = threadIdx.x;
    const int32_t slot0 = base & ~(group - 1);
    const int32_t room = tile - (base - slot0);
    const int32_t want = range_end - base < room ? range_end - base : room;
    const RowWindow w = load_row_window(a, row_lb, base, want, s_win);
    const int32_t end = base + w.cnt;

    for (int q = tid; q < tile; q += kBlock) {
        TileEntry e;
        e.col = 0; e.val = 0.0f; e.row = 0; e.meta = 0;
        const int32_t p = slot0 + q;
        if (p >= base && p < end) {
            const int32_t wi = last_row_at_or_before(s_win, w.n_first, w.n_last, p);
            const int32_t p_begin = s_win[wi];
            const int32_t p_end = s_win[wi + 1];
            const int32_t left = p_end - 1 - p;
            int32_t meta = kMetaValid | (left < kMetaSpanMask ? left : kMetaSpanMask);
            // a run starts at the row's first entry and at the chunk's first position
            if (p == p_begin || p == base) meta |= kMetaRowStart;
            if ((p_begin >> log2_group) == ((p_end - 1) >> log2_group)) meta |= kMetaPlain;
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
// the first lane of every run writes.  Lanes past the end of A contribute +0.
//   lane = (slot*G + member)*LC + chunk ; member <-> consecutive positions
// kParDepth steps are issued together so that several gathered rows of B are
// in flight per lane.
constexpr int kParDepth = 4;

template <int G, int LC, int VEC, bool OFF32>
__global__ __launch_bounds__(kBlock) void nnz_parallel_kernel(SpmmArgs a, int tile)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    TileEntry* s_tile = reinterpret_cast<TileEntry*>(s_raw);
    __shared__ int32_t s_win[kWindowCap + 1];
    constexpr int ENTRIES_PER_WAVE = kWave / LC;  // positions one wave covers per step
    constexpr int ENTRIES_PER_STEP = ENTRIES_PER_WAVE * kWavesPerBlock;

    const int32_t nnz = a.rowptr[a.M];
    const PosRange pr = my_positions(nnz, tile);
    if (pr.begin >= pr.end) return;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int entry_lane = lane / LC;  // = slot*G + member
    const int member = entry_lane % G;
    const int chunk = lane % LC;
    const int64_t N = a.N;
    const int steps = tile / ENTRIES_PER_STEP;  // host keeps this a multiple of kParDepth

    int32_t row_lb = last_row_at_or_before(a.rowptr, 0, (int32_t)a.M - 1, (int32_t)pr.begin);
    for (int32_t base = (int32_t)pr.begin; base < (int32_t)pr.end;) {
        base += stage_tile(a, base, (int32_t)pr.end, tile, G, a.log2_group, s_tile, s_win, row_lb);
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
                    const bool valid = (e[u].meta & kMetaValid) != 0;
                    int span = e[u].meta & kMetaSpanMask;
                    span = span < G - 1 - member ? span : G - 1 - member;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) x[u].v[i] = group_seg_sum<G, LC>(e[u].val * x[u].v[i], span);
                    const bool head = valid && (member == 0 || (e[u].meta & kMetaRowStart));
                    if (head && k_ok) write_out<VEC>(a, e[u].row, k, (e[u].meta & kMetaPlain) != 0, x[u]);
                }
            }
        }
        __syncthreads();  // tile fully consumed before it is overwritten
    }
}

// Rows that will receive atomic adds (their positions straddle an aligned
// block of `group` positions) and rows without stored entries are set to +0.
// thread = (row_lane, chunk); chunk lanes stride over the row's columns.
template <int VEC>
__global__ __launch_bounds__(kBlock) void zero_rows_kernel(SpmmArgs a, int lcz)
{
    const int chunk = threadIdx.x % lcz;
    const int row_lane = threadIdx.x / lcz;
    const int rows_per_block = kBlock / lcz;
    const int64_t row = (int64_t)blockIdx.x * rows_per_block + row_lane;
    if (row >= a.M) return;
    const int32_t p_begin = a.rowptr[row];
    const int32_t p_end = a.rowptr[row + 1];
    const bool plain = p_end > p_begin && (p_begin >> a.log2_group) == ((p_end - 1) >> a.log2_group);
    if (plain) return;
    Vec<VEC> z;
    z.zero();
    float* __restrict__ dst = a.C + row * a.N;
    for (int64_t k = (int64_t)chunk * VEC; k < a.N; k += (int64_t)lcz * VEC) store_vec<VEC>(dst + k, z);
}

namespace {

struct LaunchNnzParallel {
    const SpmmArgs& a;
    int compute_units;
    int64_t nnz_hint;
    bool off32;
    hipStream_t s;
    template <int G, int LC, int VEC>
    void operator()() const
    {
        // one step covers 4*64/LC positions; keep kParDepth steps per batch
        constexpr int per_batch = (kWave / LC) * kWavesPerBlock * kParDepth;
        constexpr int tile = per_batch > 1024 ? per_batch : 1024;
        constexpr int smem = tile * (int)sizeof(TileEntry);
        static const int per_cu_32 = resident_per_cu(nnz_parallel_kernel<G, LC, VEC, true>, smem);
        static const int per_cu_64 = resident_per_cu(nnz_parallel_kernel<G, LC, VEC, false>, smem);
        const int grid = persistent_grid(off32 ? per_cu_32 : per_cu_64, compute_units, nnz_hint, tile);
        if (off32)
            hipLaunchKernelGGL((nnz_parallel_kernel<G, LC, VEC, true>), dim3(grid), dim3(kBlock), smem, s, a, tile);
        else
            hipLaunchKernelGGL((nnz_parallel_kernel<G, LC, VEC, false>), dim3(grid), dim3(kBlock), smem, s, a, tile);
    }
};

}  // namespace

hipError_t launch_nnz_parallel(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, hipStream_t s)
{
    if (!dispatch_group(a.group, lc, vec, LaunchNnzParallel{a, compute_units, nnz_hint, offsets_fit_32(a), s}))
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_nnz_zero_rows(const SpmmArgs& a, int vec, hipStream_t s)
{
    int64_t chunks = (a.N + vec - 1) / vec;
    int lcz = 1;
    while (lcz < 64 && lcz < chunks) lcz *= 2;
    const int rows_per_block = kBlock / lcz;
    const int64_t grid = (a.M + rows_per_block - 1) / rows_per_block;
    switch (vec) {
        case 4: hipLaunchKernelGGL((zero_rows_kernel<4>), dim3((unsigned)grid), dim3(kBlock), 0, s, a, lcz); break;
        case 2: hipLaunchKernelGGL((zero_rows_kernel<2>), dim3((unsigned)grid), dim3(kBlock), 0, s, a, lcz); break;
        case 1: hipLaunchKernelGGL((zero_rows_kernel<1>), dim3((unsigned)grid), dim3(kBlock), 0, s, a, lcz); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sgap
