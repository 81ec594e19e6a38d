// Pieces shared by the two nnz-balanced kernels: handing out tiles of stored
// entries, finding the rows a tile touches, and the write-back rule.
//
// Merge rule (both strategies and the zeroing pass): positions are grouped in
// aligned blocks of `group` positions.  A non-empty row whose positions all
// fall in one block is produced by exactly one writer and is stored plainly;
// every other row is zeroed by zero_rows_kernel beforehand and receives
// partial sums through fp32 atomic adds.
#pragma once
#include "sgap_common.hpp"

namespace sgap {

constexpr int kWindowCap = 1024;  // rowptr window entries cached in LDS

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

// Stored entries are handed to workgroups in contiguous runs of whole tiles,
// so that each workgroup walks rowptr forward only once.
struct PosRange { int64_t begin, end; };
__device__ __forceinline__ PosRange my_positions(int32_t nnz, int tile)
{
    const int64_t tiles = ((int64_t)nnz + tile - 1) / tile;
    const int64_t per = (tiles + gridDim.x - 1) / gridDim.x;
    PosRange r;
    r.begin = (int64_t)blockIdx.x * per * tile;
    r.end = r.begin + per * tile;
    if (r.begin > nnz) r.begin = nnz;
    if (r.end > nnz) r.end = nnz;
    return r;
}

template <int VEC>
__device__ __forceinline__ void write_out(const SpmmArgs& a, int32_t row, int64_t k, bool plain,
                                          const Vec<VEC>& x)
{
    float* __restrict__ dst = a.C + (int64_t)row * a.N + k;
    if (plain) store_vec<VEC>(dst, x); else atomic_add_vec<VEC>(dst, x);
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

inline int persistent_grid(int per_cu, int compute_units, int64_t nnz_hint, int tile)
{
    int64_t grid = (int64_t)per_cu * compute_units;
    if (nnz_hint >= 0) {
        const int64_t tiles = (nnz_hint + tile - 1) / tile;
        if (tiles < grid) grid = tiles > 0 ? tiles : 1;
    }
    return (int)grid;
}

}  // namespace sgap
