// Nnz-balanced schedule: the unit of work is a stored entry of A (the paper's
// first atomic-parallelism family, <x nnz, y col>, Section 3.2).  Stored
// entries are cut into tiles of kTile positions; a workgroup stages a tile's
// (column, value, row, meta) records in LDS and then lets its lanes combine
// them.  The row of a position is found by searching rowptr, as in the paper's
// Listings 1 and 2, but only inside the tile's window of rows, which is kept
// in LDS when it fits.
//
// Merge rule shared by both strategies and the zeroing pass: positions are
// grouped in aligned blocks of `group` positions.  A non-empty row whose
// positions all fall in one block is produced by exactly one writer and is
// stored plainly; every other row is zeroed by zero_rows_kernel beforehand
// and receives partial sums through fp32 atomic adds.
#include "sgap_common.hpp"
#include "sgap_lane_ops.hpp"

namespace sgap {

constexpr int kTile = 1024;        // stored entries per LDS tile
constexpr int kWindowCap = 1024;   // rowptr window entries cached in LDS

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

// Largest r in [lo, hi] with rowptr[r] <= pos  (rowptr[lo] <= pos is given).
__device__ __forceinline__ int32_t last_row_at_or_before(const int32_t* __restrict__ rowptr, int32_t lo,
                                                         int32_t hi, int32_t pos)
{
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo + 1) / 2;
        if (rowptr[mid] <= pos) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Stage tile `tile` into LDS.  `row_lb` is any row with rowptr[row_lb] <= the
// tile's first position; on return it is the row of the tile's last position
// (a valid lower bound for the next tile).  Block-uniform control flow.
__device__ __forceinline__ void stage_tile(const SpmmArgs& a, int32_t nnz, int64_t tile, int log2_group,
                                           TileEntry* __restrict__ s_tile, int32_t* __restrict__ s_win,
                                           int32_t& row_lb)
{
    const int tid = threadIdx.x;
    const int32_t base = (int32_t)(tile * kTile);
    const int32_t cnt = nnz - base < kTile ? nnz - base : kTile;
    const int32_t last = base + cnt - 1;
    const int32_t M = (int32_t)a.M;

    // Walk rowptr forward from row_lb in chunks of kBlock entries: count rows
    // that start at or before the tile's first / last position and keep the
    // values in the LDS window.  rowptr[M] = nnz > last ends the walk.
    int32_t n_first = 0, n_last = 0;
    if (tid == 0) s_win[0] = a.rowptr[row_lb];
    for (int32_t off = 1;; off += kBlock) {
        const int64_t r = (int64_t)row_lb + off + tid;
        const int32_t v = r <= M ? a.rowptr[r] : 0x7fffffff;
        if (off + tid <= kWindowCap) s_win[off + tid] = v;
        const int c_last = __syncthreads_count(v <= last);
        const int c_first = __syncthreads_count(v <= base);
        n_first += c_first;
        n_last += c_last;
        if (c_last < kBlock) break;
    }
    const int32_t r_first = row_lb + n_first;
    const int32_t r_last = row_lb + n_last;
    // window index of row r is r - row_lb; entries up to r_last+1 are needed
    const bool win_in_lds = (n_last + 1) <= kWindowCap;

    for (int q = tid; q < kTile; q += kBlock) {
        TileEntry e;
        e.col = 0; e.val = 0.0f; e.row = 0; e.meta = 0;
        if (q < cnt) {
            const int32_t p = base + q;
            int32_t row, p_begin, p_end;
            if (win_in_lds) {
                const int32_t w = last_row_at_or_before(s_win, n_first, n_last, p);
                row = row_lb + w;
                p_begin = s_win[w];
                p_end = s_win[w + 1];
            } else {
                row = last_row_at_or_before(a.rowptr, r_first, r_last, p);
                p_begin = a.rowptr[row];
                p_end = a.rowptr[row + 1];
            }
            const int32_t left = p_end - 1 - p;
            int32_t meta = kMetaValid | (left < kMetaSpanMask ? left : kMetaSpanMask);
            if (p == p_begin) meta |= kMetaRowStart;
            if ((p_begin >> log2_group) == ((p_end - 1) >> log2_group)) meta |= kMetaPlain;
            e.col = a.colidx[p];
            e.val = a.vals[p];
            e.row = row;
            e.meta = meta;
        }
        s_tile[q] = e;
    }
    row_lb = r_last;
    __syncthreads();
}

// Tiles are handed to workgroups in contiguous runs so that each workgroup
// walks rowptr forward only once.
struct TileRange { int64_t begin, end; };
__device__ __forceinline__ TileRange my_tiles(int32_t nnz)
{
    const int64_t tiles = ((int64_t)nnz + kTile - 1) / kTile;
    const int64_t per = (tiles + gridDim.x - 1) / gridDim.x;
    TileRange r;
    r.begin = (int64_t)blockIdx.x * per;
    r.end = r.begin + per < tiles ? r.begin + per : tiles;
    return r;
}

template <int VEC>
__device__ __forceinline__ void write_out(const SpmmArgs& a, int32_t row, int64_t k, bool plain,
                                          const Vec<VEC>& x)
{
    float* __restrict__ dst = a.C + (int64_t)row * a.N + k;
    if (plain) store_vec<VEC>(dst, x); else atomic_add_vec<VEC>(dst, x);
}

// {<1 nnz, c col>, r} with r = G (Section 6.2, the "1 nnz" listing; Listing 2
// is its G = 32 instance): a lane multiplies ONE stored entry by its column
// chunk; the G members of a group then run a segmented sum keyed by row and
// the first lane of every run writes.  Lanes past the end of A contribute +0.
//   lane = (slot*G + member)*LC + chunk ; member <-> consecutive positions
template <int G, int LC, int VEC>
__global__ __launch_bounds__(kBlock) void nnz_parallel_kernel(SpmmArgs a)
{
    __shared__ TileEntry s_tile[kTile];
    __shared__ int32_t s_win[kWindowCap + 1];
    constexpr int ENTRIES_PER_WAVE = kWave / LC;  // positions one wave covers per step
    constexpr int STEPS = kTile / (ENTRIES_PER_WAVE * kWavesPerBlock);
    static_assert(STEPS >= 1, "tile too small");

    const int32_t nnz = a.rowptr[a.M];
    const TileRange tr = my_tiles(nnz);
    if (tr.begin >= tr.end) return;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int entry_lane = lane / LC;  // = slot*G + member
    const int member = entry_lane % G;
    const int chunk = lane % LC;
    const int64_t N = a.N;

    int32_t row_lb = last_row_at_or_before(a.rowptr, 0, (int32_t)a.M - 1, (int32_t)(tr.begin * kTile));
    for (int64_t tile = tr.begin; tile < tr.end; ++tile) {
        stage_tile(a, nnz, tile, a.log2_group, s_tile, s_win, row_lb);
        for (int64_t k0 = 0; k0 < N; k0 += (int64_t)LC * VEC) {
            const int64_t k = k0 + (int64_t)chunk * VEC;
            const bool k_ok = k < N;
#pragma unroll 2
            for (int step = 0; step < STEPS; ++step) {
                const int q = (step * kWavesPerBlock + wave) * ENTRIES_PER_WAVE + entry_lane;
                const TileEntry e = s_tile[q];
                const bool valid = (e.meta & kMetaValid) != 0;
                Vec<VEC> x;
                x.zero();
                if (valid && k_ok) x.fma(e.val, load_vec<VEC>(a.B + (int64_t)e.col * N + k));
                int span = e.meta & kMetaSpanMask;
                span = span < G - 1 - member ? span : G - 1 - member;
#pragma unroll
                for (int i = 0; i < VEC; ++i) x.v[i] = group_seg_sum<G, LC>(x.v[i], span);
                const bool head = valid && (member == 0 || (e.meta & kMetaRowStart));
                if (head && k_ok) write_out<VEC>(a, e.row, k, (e.meta & kMetaPlain) != 0, x);
            }
        }
        __syncthreads();  // tile fully consumed before it is overwritten
    }
}

// {<g nnz, c col>, 1} (Section 6.1, the "g nnz" listing): a lane walks `group`
// consecutive stored entries serially and flushes its register whenever the
// row ends or its share ends (conditional reduction).
//   thread = entry_lane*LC + chunk over the whole workgroup
template <int LC, int VEC>
__global__ __launch_bounds__(kBlock) void nnz_serial_kernel(SpmmArgs a)
{
    __shared__ TileEntry s_tile[kTile];
    __shared__ int32_t s_win[kWindowCap + 1];
    constexpr int ENTRY_LANES = kBlock / LC;

    const int32_t nnz = a.rowptr[a.M];
    const TileRange tr = my_tiles(nnz);
    if (tr.begin >= tr.end) return;

    const int entry_lane = threadIdx.x / LC;
    const int chunk = threadIdx.x % LC;
    const int64_t N = a.N;
    const int G = a.group;
    const int per_step = ENTRY_LANES * G;  // positions the workgroup covers per step

    int32_t row_lb = last_row_at_or_before(a.rowptr, 0, (int32_t)a.M - 1, (int32_t)(tr.begin * kTile));
    for (int64_t tile = tr.begin; tile < tr.end; ++tile) {
        stage_tile(a, nnz, tile, a.log2_group, s_tile, s_win, row_lb);
        for (int64_t k0 = 0; k0 < N; k0 += (int64_t)LC * VEC) {
            const int64_t k = k0 + (int64_t)chunk * VEC;
            if (k < N) {
                for (int q0 = entry_lane * G; q0 < kTile; q0 += per_step) {
                    Vec<VEC> acc;
                    acc.zero();
                    for (int j = 0; j < G; ++j) {
                        const TileEntry e = s_tile[q0 + j];
                        if (!(e.meta & kMetaValid)) break;
                        acc.fma(e.val, load_vec<VEC>(a.B + (int64_t)e.col * N + k));
                        if ((e.meta & kMetaSpanMask) == 0 || j == G - 1) {
                            write_out<VEC>(a, e.row, k, (e.meta & kMetaPlain) != 0, acc);
                            acc.zero();
                        }
                    }
                }
            }
        }
        __syncthreads();
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
    int grid;
    hipStream_t s;
    template <int G, int LC, int VEC>
    void operator()() const
    {
        hipLaunchKernelGGL((nnz_parallel_kernel<G, LC, VEC>), dim3(grid), dim3(kBlock), 0, s, a);
    }
};
struct LaunchNnzSerial {
    const SpmmArgs& a;
    int grid;
    hipStream_t s;
    template <int G, int LC, int VEC>
    void operator()() const
    {
        hipLaunchKernelGGL((nnz_serial_kernel<LC, VEC>), dim3(grid), dim3(kBlock), 0, s, a);
    }
};
}  // namespace

hipError_t launch_nnz_parallel(const SpmmArgs& a, int lc, int vec, int grid, hipStream_t s)
{
    if (!dispatch_group(a.group, lc, vec, LaunchNnzParallel{a, grid, s})) return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_nnz_serial(const SpmmArgs& a, int lc, int vec, int grid, hipStream_t s)
{
    if (!dispatch_lc<1>(lc, vec, LaunchNnzSerial{a, grid, s})) return hipErrorInvalidValue;
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
