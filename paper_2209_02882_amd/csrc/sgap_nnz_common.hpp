// Pieces shared by the two nnz-balanced kernels: handing out tiles of stored
// entries, finding the rows a tile touches, and the write-back rule.
//
// Merge rule (both strategies and the zeroing pass): positions are grouped in
// aligned "merge blocks" of 2^merge_log2 positions.  A non-empty row whose
// positions all fall in one merge block is written exactly once with a plain
// store; every other row is zeroed by zero_rows_kernel beforehand and receives
// partial sums through global fp32 atomic adds.
//   direct mode: merge block = the `group` positions of one segment group /
//     lane; every partial sum of a group goes straight to global memory.
//   tile mode:   merge block = one tile of positions.  Partial sums of rows
//     that lie inside the tile are first combined in LDS accumulators (LDS
//     atomic adds) and written once; only rows that cross a tile boundary use
//     global atomics.  Global fp32 atomics are far more expensive than loads
//     on this chip, so tile mode is used whenever the accumulators fit.
#pragma once
#include "sgap_common.hpp"
#include "sgap_tile_deal.hpp"

namespace sgap {

constexpr int kWindowCap = 1024;              // rowptr window entries cached in LDS
constexpr int kMergeLdsBudget = 34 * 1024;    // bytes of LDS accumulators tile mode may take
// Small groups at wide N need one accumulator per one or two positions, far more than that budget.  Going
// without tile mode there means a global atomic add per stored entry (or two), tens of times slower than
// anything else in the space (Section 6.2 shows that point, its Listing 1, as the one to get away from), so
// such points may take most of a compute unit's LDS (one workgroup per compute unit is resident then), and
// what still does not fit runs with fewer chunk lanes per entry (more passes over the columns).
constexpr int kMergeLdsLimit = 137 * 1024;
constexpr int kParTile = 1024;                // positions per tile of the parallel strategy
constexpr int kTileRowBatch = 256;            // tiles whose first rows a workgroup looks up at once

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

// First index in sorted s[0..n) whose value exceeds pos (n if none).
__device__ __forceinline__ int32_t first_above(const int32_t* __restrict__ s, int32_t n, int32_t pos)
{
    int32_t lo = 0, hi = n;
    while (lo < hi) {
        const int32_t mid = (lo + hi) / 2;
        if (s[mid] <= pos) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// The rows touched by a chunk of positions, relative to row_lb: window index
// w stands for row row_lb + w, and s_win[w] = rowptr[min(row_lb + w, M)] for
// 0 <= w <= kWindowCap.
struct RowWindow {
    int32_t n_first;  // window index of the row holding the chunk's first position
    int32_t n_last;   // window index of the row holding the chunk's last position
    int32_t cnt;      // positions in the chunk (may be cut short, see below)
};

// Copy kWindowCap+1 entries of rowptr, starting at row_lb (a row with
// rowptr[row_lb] <= first_pos), into the LDS window and locate the rows of the
// chunk [first_pos, first_pos + want).  When the chunk reaches beyond the
// window (long runs of rows without stored entries) it is cut back to the
// positions the window's rows hold.  The cut falls on a row boundary, so no
// row is split by it and the merge rule is unaffected.  If not even first_pos
// lies inside the window, row_lb is first moved up by bisecting rowptr.
// Block-uniform; every thread gets the same result; s_win is ready on return.
__device__ __forceinline__ RowWindow load_row_window(const SpmmArgs& a, int32_t& row_lb, int32_t first_pos,
                                                     int32_t want, int32_t* __restrict__ s_win)
{
    const int32_t M = (int32_t)a.M;
    while (true) {
        for (int i = threadIdx.x; i <= kWindowCap; i += kBlock) {
            const int64_t r = (int64_t)row_lb + i;
            s_win[i] = a.rowptr[r <= M ? r : M];
        }
        __syncthreads();
        const int32_t top = s_win[kWindowCap];
        if (top > first_pos) break;
        // more than kWindowCap rows without entries before first_pos's row
        __syncthreads();  // everyone has read `top` before the window is reloaded
        row_lb = last_row_at_or_before(a.rowptr, row_lb + kWindowCap, M - 1, first_pos);
    }
    RowWindow w;
    const int32_t top = s_win[kWindowCap];  // > first_pos
    w.cnt = top <= first_pos + want - 1 ? top - first_pos : want;
    // rows at window index < first_above(...) start at or before the position
    w.n_first = first_above(s_win, kWindowCap + 1, first_pos) - 1;
    w.n_last = first_above(s_win, kWindowCap + 1, first_pos + w.cnt - 1) - 1;
    return w;
}

// Cut the plain window of a tile (s_win[r] = rowptr[row_lb + r], r <= kWindowCap, with s_win[kWindowCap] >=
// tile_end, and row_lb the row of the tile's first position) down, in place, to the rows with entries that start
// below tile_end: on return s_win[0 .. n] holds their first positions (and the end of the last), s_row[0 .. n)
// their rows; n is returned.  A kept row moves to a slot at or in front of its own, every round reads its kBlock
// slots before any is written, and a slot that a later round still reads is only ever overwritten with the value
// it holds (the next row with entries starts where this one ends).  Block-uniform; two barriers per kBlock rows.
__device__ __forceinline__ int32_t compact_window(int32_t* __restrict__ s_win, int32_t* __restrict__ s_row,
                                                  int32_t row_lb, int32_t tile_end, int32_t* __restrict__ s_wave)
{
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    int32_t n = 0;
    for (int32_t r0 = 0;; r0 += kBlock) {
        const int32_t r = r0 + tid;
        int32_t lo = 0x7fffffff, hi = 0x7fffffff;
        if (r < kWindowCap) {
            lo = s_win[r];
            hi = s_win[r + 1];
        }
        const bool keep = hi > lo && lo < tile_end;
        const unsigned long long mask = __ballot(keep);
        if (lane == 0) s_wave[wave] = (int32_t)__popcll(mask);
        // rows are looked at in order: once one starts at or beyond tile_end (or the window ends) no later one counts
        const bool done = __syncthreads_or(lo >= tile_end);
        int32_t before = 0, total = 0;
#pragma unroll
        for (int v = 0; v < kWavesPerBlock; ++v) {
            const int32_t c = s_wave[v];
            if (v < wave) before += c;
            total += c;
        }
        if (keep) {
            const int32_t j = n + before + (int32_t)__popcll(mask & ((1ull << lane) - 1ull));
            s_win[j] = lo;
            s_win[j + 1] = hi;
            s_row[j] = row_lb + r;
        }
        n += total;
        __syncthreads();  // written before the next round reads on (or the caller does); s_wave is free again
        if (done) break;
    }
    return n;
}

// A window of the rows WITH stored entries that the tile [tile_start, tile_end) touches, for tiles whose rows do
// not fit the plain window (long runs of rows without entries, as at the sparse end of an R-MAT matrix: a tile of
// 1,024 entries there spans up to 9,000 rows).  The workgroup scans rowptr from row_lb (the row of tile_start) on,
// 256 rows at a time, and keeps (first position, row) of every row that has entries below tile_end; such rows
// start at distinct positions, one of them at or before tile_start and the others inside the tile, so there are
// no more of them than the tile has positions, and the arrays are sized for that.  Returns the number of rows kept;
// s_win[0 .. n] and s_row[0 .. n) are ready on return.  Block-uniform.
__device__ __forceinline__ int32_t load_compact_window(const SpmmArgs& a, int32_t row_lb, int32_t tile_end,
                                                       int32_t* __restrict__ s_win, int32_t* __restrict__ s_row,
                                                       int32_t* __restrict__ s_wave)
{
    const int32_t M = (int32_t)a.M;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    int32_t n = 0;
    for (int64_t r0 = row_lb;; r0 += kBlock) {
        const int64_t r = r0 + tid;
        int32_t lo = 0x7fffffff, hi = 0x7fffffff;
        if (r < M) {
            lo = a.rowptr[r];
            hi = a.rowptr[r + 1];
        }
        const bool keep = r < M && hi > lo && lo < tile_end;
        const unsigned long long mask = __ballot(keep);
        __syncthreads();  // s_wave is free again
        if (lane == 0) s_wave[wave] = (int32_t)__popcll(mask);
        __syncthreads();
        int32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) {
            const int32_t c = s_wave[w];
            if (w < wave) before += c;
            total += c;
        }
        if (keep) {
            const int32_t j = n + before + (int32_t)__popcll(mask & ((1ull << lane) - 1ull));
            s_win[j] = lo;
            s_row[j] = (int32_t)r;
        }
        n += total;
        // rows are looked at in order: once one starts at or beyond tile_end (or the matrix ends) no later one counts
        if (__syncthreads_or(lo >= tile_end)) break;
    }
    if (tid == 0) s_win[n] = a.rowptr[s_row[n - 1] + 1];  // where the last kept row ends (n >= 1: row_lb has entries)
    __syncthreads();
    return n;
}

// The whole workgroup looks for one row together: each round probes rowptr at
// up to kBlock evenly spaced rows and keeps the stretch between the last
// probe at or before `pos` and the next one (3 rounds for 2 M rows, where a
// single thread's bisection takes 21 dependent loads).  Returns the largest r
// in [lo, hi] with rowptr[r] <= pos (rowptr[lo] <= pos is given).
// Block-uniform; contains barriers.
__device__ __forceinline__ int32_t find_row_cooperative(const int32_t* __restrict__ rowptr, int32_t lo, int32_t hi,
                                                        int32_t pos)
{
    const int tid = threadIdx.x;
    while (lo < hi) {
        const int64_t span = (int64_t)hi - lo;
        const int64_t step = (span + kBlock - 1) / kBlock;  // >= 1
        int64_t r = (int64_t)lo + (tid + 1) * step;
        if (r > hi) r = hi;
        const int cnt = __syncthreads_count(rowptr[r] <= pos);  // probes are sorted: the first cnt hold
        if (cnt == kBlock) return hi;  // the last probe is hi itself
        int64_t next = (int64_t)lo + (cnt + 1) * step;  // first probe beyond pos
        if (next > hi) next = hi;
        if (cnt > 0) lo = (int32_t)((int64_t)lo + cnt * step);
        hi = (int32_t)next - 1;
    }
    return lo;
}

// Rows of the first positions of this workgroup's tiles number j0 .. j0+n-1
// (`deal` says which tiles those are; `tile` positions each),
// left in s_tile_row[0..n).  A workgroup with many tiles lets each thread
// bisect for one tile; one with a few searches for them together, which is
// what bounds the run time of small matrices.  Block-uniform; s_tile_row is
// ready on return.
constexpr int kFewTiles = 4;
__device__ __forceinline__ void find_tile_rows(const SpmmArgs& a, const TileDeal& deal, int64_t j0, int tile,
                                               int32_t* __restrict__ s_tile_row)
{
    const int32_t M = (int32_t)a.M;
    const int tid = threadIdx.x;
    const int64_t n = deal.mine - j0 < kTileRowBatch ? deal.mine - j0 : kTileRowBatch;
    __syncthreads();  // the previous batch's rows are no longer needed
    if (n <= kFewTiles) {
        int32_t lo = 0;
        for (int j = 0; j < (int)n; ++j) {
            lo = find_row_cooperative(a.rowptr, lo, M - 1, (int32_t)(deal.tile(j0 + j) * tile));
            if (tid == 0) s_tile_row[j] = lo;
        }
    } else if (tid < n) {
        s_tile_row[tid] =
            last_row_at_or_before(a.rowptr, 0, M - 1, (int32_t)(deal.tile(j0 + tid) * tile));
    }
    __syncthreads();
}

// One run's sum leaves the registers: a plain store when nobody else adds to the
// row, else atomic adds.  The LC chunk lanes of an entry lane whose columns lie
// inside N call this together.  They hold LC*VEC consecutive columns, VEC per
// lane; an atomic instruction whose lanes are 16 bytes apart costs four times
// one over consecutive words, so where the pass is complete (all LC lanes are
// here) the sums change hands first: in round q lane c adds column q*LC + c,
// which chunk lane (q*LC + c) / VEC holds.
template <int LC, int VEC>
__device__ __forceinline__ void write_out(const SpmmArgs& a, int32_t row, int64_t k, bool plain,
                                          const Vec<VEC>& x)
{
    float* __restrict__ dst = a.C + (int64_t)row * a.N + k;
    if (plain) {
        store_vec<VEC>(dst, x);
        return;
    }
    if constexpr (LC >= VEC && VEC > 1) {
        const int chunk = threadIdx.x % LC;
        const int64_t k0 = k - (int64_t)chunk * VEC;  // first column of this pass
        if (k0 + LC * VEC <= a.N) {                   // the same for all lanes of the pass
#pragma unroll
            for (int q = 0; q < VEC; ++q) {
                const int col = q * LC + chunk;
                float mine = 0.0f;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const float t = __shfl(x.v[v], col / VEC, LC);
                    if (col % VEC == v) mine = t;
                }
                unsafeAtomicAdd(a.C + (int64_t)row * a.N + k0 + col, mine);
            }
            return;
        }
    }
    atomic_add_vec<VEC>(dst, x);
}

// LDS accumulators of tile mode.  Slot s < nslots-1 belongs to the row whose
// first stored entry lies in the s-th aligned block of `group` positions of
// the tile and which continues past that block (at most one such row per
// block); the last slot belongs to the row that entered the chunk from the
// left.  Each slot holds `width` floats: the columns of the current pass.
struct MergeBuf {
    float* accum;          // nslots * width floats, zero between uses
    int32_t* slot_row;     // nslots, -1 = unused
    int32_t* slot_atomic;  // nslots, 1 = the row also has entries outside the chunk
    int32_t nslots;
    int32_t width;
};

__device__ __forceinline__ void merge_reset(const MergeBuf& mb)
{
    for (int i = threadIdx.x; i < mb.nslots * mb.width; i += kBlock) mb.accum[i] = 0.0f;
    for (int i = threadIdx.x; i < mb.nslots; i += kBlock) mb.slot_row[i] = -1;
}

// fp32 add into an LDS word shared with other lanes.  The LDS fp32 atomic add
// instruction retires about one lane every three clocks per compute unit on
// this chip (measured: 0.33 lane-ops/clk/CU against 14.5 for integer LDS
// atomics); a compare-and-swap loop on the integer path does the same job at
// 4.7 lane-ops/clk/CU when few lanes meet on an address, as here (a row's
// partial sums come from the two or three lanes whose shares it crosses).
__device__ __forceinline__ void lds_add_f32(float* p, float x)
{
    int* ip = reinterpret_cast<int*>(p);
    int old = *reinterpret_cast<volatile int*>(ip);
    while (true) {
        const int want = __float_as_int(__int_as_float(old) + x);
        const int seen = atomicCAS(ip, old, want);
        if (seen == old) break;
        old = seen;
    }
}

// One lane adds its partial sum of a row into the row's slot.  `owner` is set
// for the lane that holds the row's first entry inside the chunk (column
// chunk 0 only): it records which row the slot stands for.
// CAS picks the compare-and-swap loop (few lanes per address: the serial
// strategy) or the hardware's fp32 LDS atomic (many lanes of one wavefront on
// one address, where the loop would retry once per lane: the parallel strategy).
template <int VEC, bool CAS>
__device__ __forceinline__ void merge_add(const MergeBuf& mb, int32_t slot, int lane_col, const Vec<VEC>& x,
                                          bool owner, int32_t row, bool needs_atomic)
{
    float* dst = mb.accum + slot * mb.width + lane_col;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        if constexpr (CAS) lds_add_f32(dst + i, x.v[i]);
        else __hip_atomic_fetch_add(dst + i, x.v[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    if (owner) {
        mb.slot_row[slot] = row;
        mb.slot_atomic[slot] = needs_atomic ? 1 : 0;
    }
}

// After a barrier: write every used slot to C (plain store, or global atomic
// add for rows that continue outside the chunk) and clear it for the next use.
// thread = slot_lane*LC + chunk, the same column mapping as the compute phase.
// The LC lanes of a slot sit in one wavefront, so the owner lane's reset of
// slot_row cannot overtake the other lanes' reads.
template <int LC, int VEC>
__device__ __forceinline__ void merge_write_out(const SpmmArgs& a, const MergeBuf& mb, int64_t k, bool k_ok)
{
    constexpr int SLOT_LANES = kBlock / LC;
    const int chunk = threadIdx.x % LC;
    for (int s = threadIdx.x / LC; s < mb.nslots; s += SLOT_LANES) {
        const int32_t row = mb.slot_row[s];
        if (row < 0) continue;
        if (mb.slot_atomic[s]) {
            // atomic adds over consecutive words: an instruction whose lanes are 16 bytes apart
            // costs four times as much, and out of LDS any lane can take any column
            float* src = mb.accum + s * mb.width;
            const int64_t k0 = k - (int64_t)chunk * VEC;  // first column of this pass
#pragma unroll
            for (int q = 0; q < VEC; ++q) {
                const int col = q * LC + chunk;
                const float x = src[col];
                src[col] = 0.0f;
                if (k0 + col < a.N) unsafeAtomicAdd(a.C + (int64_t)row * a.N + k0 + col, x);
            }
        } else {
            float* src = mb.accum + s * mb.width + chunk * VEC;
            Vec<VEC> x;
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                x.v[i] = src[i];
                src[i] = 0.0f;
            }
            if (k_ok) store_vec_stream<VEC>(a.C + (int64_t)row * a.N + k, x);
        }
        if (chunk == 0) mb.slot_row[s] = -1;
    }
}

// Host side: workgroups of a kernel instance one compute unit can hold, and
// the persistent grid built from it.
template <typename K>
inline int resident_per_cu(K kernel, int smem)
{
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kernel, kBlock, smem) != hipSuccess || n < 1) n = 1;
    return n;
}

// More dynamic LDS than the default limit of a launch (64 KB with the kernel's static LDS) has to be asked for.
// `asked` is the caller's record, per kernel instance, of the most it has asked for so far: an instance runs
// with different amounts (the slots of the merge rule depend on the group size), and the limit only grows.
template <typename K>
inline void ensure_dynamic_lds(K kernel, int smem, int& asked)
{
    if (smem <= 32 * 1024 || smem <= asked) return;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, smem) ==
        hipSuccess)
        asked = smem;
}

inline int persistent_grid(int per_cu, int compute_units, int64_t nnz_hint, int tile)
{
    int64_t grid = (int64_t)per_cu * compute_units;
    if (grid >= 8) grid -= grid % 8;  // whole rounds of the 8 dies, see TileDeal
    if (nnz_hint >= 0) {
        // a matrix with no more tiles than that gets one workgroup per tile
        const int64_t tiles = (nnz_hint + tile - 1) / tile;
        if (tiles <= grid) grid = tiles > 0 ? tiles : 1;
    }
    return (int)grid;
}

}  // namespace sgap
