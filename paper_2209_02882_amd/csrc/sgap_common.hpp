// Shared declarations of the SpMM kernels: argument block, per-lane column
// vectors (the paper's coarsening factor c = VEC dense columns per lane) and
// the host-side launch entry points of each kernel family.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sgap {

constexpr int kWave = 64;          // wavefront size on gfx950
constexpr int kBlock = 256;        // threads per workgroup (4 waves)
constexpr int kWavesPerBlock = kBlock / kWave;

struct SpmmArgs {
    int64_t M, K, N;
    const int32_t* __restrict__ rowptr;
    const int32_t* __restrict__ colidx;
    const float* __restrict__ vals;
    const float* __restrict__ B;
    float* __restrict__ C;
    int log2_group;   // log2(group_size)
    int group;        // group_size
};

// A third-order tensor as compressed sparse fibers (first index dense) and the dense operands of MTTKRP.
struct MttkrpArgs {
    int64_t I, K, L, J;
    const int32_t* __restrict__ fptr;
    const int32_t* __restrict__ fidx;
    const int32_t* __restrict__ eptr;
    const int32_t* __restrict__ eidx;
    const float* __restrict__ vals;
    const float* __restrict__ X1;
    const float* __restrict__ X2;
    float* __restrict__ Y;
};

// Rows another kernel produces: when *count <= max_rows, rows of at least
// min_len stored entries are neither computed nor written by the kernel that
// is handed this.  count = nullptr: no row is left out.
struct RowSkip {
    const uint32_t* __restrict__ count;
    uint32_t max_rows;
    int32_t min_len;
};

// How the (row block x column tile) work items of a row-split launch are
// laid over the grid.  The 8 accelerator dies (XCDs) of the chip each have a
// private L2 and receive workgroups round-robin (workgroup b runs on XCD
// b % 8), so item = (b % 8) * items_per_xcd + b / 8 hands every XCD one
// contiguous run of the column-tile-major item order: one column tile and a
// contiguous range of rows at a time, which keeps the rows of B it gathers
// resident in its own L2.
struct TileSched {
    int64_t row_blocks;     // number of row blocks
    int64_t items;          // row_blocks * col_tiles
    int64_t items_per_xcd;  // ceil(items / xcds)
    int32_t col_tiles;      // number of column tiles
    int32_t tile_cols;      // columns per tile (multiple of VEC)
    int32_t xcds;           // 8, or 1 to switch the remapping off
};

template <int VEC>
struct Vec {
    float v[VEC];
    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = 0.0f;
    }
    __device__ __forceinline__ void fma(float a, const Vec& b)
    {
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] = __builtin_fmaf(a, b.v[i], v[i]);
    }
};

// VEC consecutive floats starting at an address aligned to VEC*4 bytes.
template <int VEC>
__device__ __forceinline__ Vec<VEC> load_vec(const float* __restrict__ p)
{
    Vec<VEC> r;
    if constexpr (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
    } else if constexpr (VEC == 2) {
        const float2 t = *reinterpret_cast<const float2*>(p);
        r.v[0] = t.x; r.v[1] = t.y;
    } else {
        r.v[0] = *p;
    }
    return r;
}

template <int VEC>
__device__ __forceinline__ void store_vec(float* __restrict__ p, const Vec<VEC>& r)
{
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(r.v[0], r.v[1], r.v[2], r.v[3]);
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2*>(p) = make_float2(r.v[0], r.v[1]);
    } else {
        *p = r.v[0];
    }
}

// Streaming accesses: data touched once (A going in, C going out) should not
// displace the rows of B that the L2 keeps for reuse.
template <typename T>
__device__ __forceinline__ T load_stream(const T* __restrict__ p)
{
    return __builtin_nontemporal_load(p);
}

typedef float native_f4 __attribute__((ext_vector_type(4)));
typedef float native_f2 __attribute__((ext_vector_type(2)));

template <int VEC>
__device__ __forceinline__ void store_vec_stream(float* __restrict__ p, const Vec<VEC>& r)
{
    if constexpr (VEC == 4) {
        native_f4 t = {r.v[0], r.v[1], r.v[2], r.v[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<native_f4*>(p));
    } else if constexpr (VEC == 2) {
        native_f2 t = {r.v[0], r.v[1]};
        __builtin_nontemporal_store(t, reinterpret_cast<native_f2*>(p));
    } else {
        __builtin_nontemporal_store(r.v[0], p);
    }
}

// Address of B[col, k..): with OFF32 every byte offset into B fits 32 bits and
// col, N*4 fit 24 bits, so one 24-bit multiply-add forms the offset and the
// load uses the uniform base pointer plus a 32-bit lane offset.
template <bool OFF32>
struct BRow {
    const char* __restrict__ base;  // B as bytes
    uint32_t row_bytes;             // N * 4          (OFF32)
    uint32_t k_bytes;               // k * 4          (OFF32)
    int64_t N;                      // row stride     (!OFF32)
    int64_t k;
    __device__ __forceinline__ BRow(const float* B, int64_t n, int64_t k_)
        : base(reinterpret_cast<const char*>(B)), row_bytes((uint32_t)(n * 4)), k_bytes((uint32_t)(k_ * 4)), N(n), k(k_)
    {
    }
    __device__ __forceinline__ const float* at(int32_t col) const
    {
        if constexpr (OFF32) {
            const uint32_t off = __umul24((uint32_t)col, row_bytes) + k_bytes;
            return reinterpret_cast<const float*>(base + off);
        } else {
            return reinterpret_cast<const float*>(base) + ((int64_t)col * N + k);
        }
    }
};

inline bool offsets_fit_32(const SpmmArgs& a)
{
    return a.K <= (1 << 24) && a.N * 4 < (1 << 24) && a.K * a.N * 4 <= 0xffffffffLL;
}

// Cross-group merge: hardware fp32 atomic add (no return value needed).
template <int VEC>
__device__ __forceinline__ void atomic_add_vec(float* __restrict__ p, const Vec<VEC>& r)
{
#pragma unroll
    for (int i = 0; i < VEC; ++i) unsafeAtomicAdd(p + i, r.v[i]);
}

// How an nnz-balanced kernel cuts the stored entries: tile = positions per LDS
// tile, merge = tile mode of the merge rule, merge_log2 = log2 of the merge
// block the zeroing pass must assume (tile in tile mode, group otherwise),
// lc = chunk lanes per stored entry the kernel is to run with (the plan may
// narrow the layout it was asked about so that the accumulators fit the LDS).
struct NnzPlan {
    int tile;
    bool merge;
    int merge_log2;
    int lc;
};
NnzPlan plan_nnz_serial(int group, int lc, int vec, int64_t nnz_hint, int compute_units, int forced_tile);
NnzPlan plan_nnz_parallel(int group, int lc, int vec);
// ---- host-side launchers, one per kernel family (defined in the .hip files)
// lc = chunk lanes per row (power of two), vec = columns per lane (1, 2, 4).
// g = lanes per row (1 for the serial strategy), rows_per_slot = rows a group
// works through per work item (consecutive rows, or every slots-th row of the
// block when `interleave` is set), tile_cols = columns per work item, xcds = 8
// or 1, compute_units = CUs of the device; persistent = launch only as many
// workgroups as fit the chip and let each walk several items (else one
// workgroup per item); block = threads per workgroup (128, 256 or 512).
hipError_t launch_row_split(const SpmmArgs& a, int g, int lc, int vec, int rows_per_slot, bool interleave,
                            int tile_cols, int xcds, int compute_units, bool persistent, int block, hipStream_t s);
// the same with g lanes per row reducing in sub-groups of r < g lanes whose sums
// are merged with atomics; C must have been zeroed (launch_nnz_zero_rows, -1)
hipError_t launch_row_split_partial(const SpmmArgs& a, int g, int r, int lc, int vec, int rows_per_slot,
                                    int tile_cols, int xcds, int compute_units, bool persistent, int block,
                                    hipStream_t s);
// the row-split launch with rows of at least min_len stored entries taken out and
// produced window by window of about window_bytes of B (sgap_panels.hip); vec must be 4;
// wave_vec > 0: the other rows by launch_wave_rows with that many columns per lane and rows_per_slot rows per wavefront;
// workspace = device memory of spmm_panels_workspace_bytes(K, N, window_bytes, cap) bytes
// for a list of up to cap long rows (more long rows than that: the row-split kernel takes every row)
hipError_t launch_row_split_panels(const SpmmArgs& a, int g, int lc, int vec, int rows_per_slot, bool interleave,
                                   int tile_cols, int xcds, int compute_units, bool persistent, int block,
                                   int wave_vec, int32_t min_len, int64_t window_bytes, void* workspace, int64_t cap,
                                   hipStream_t s);
int64_t spmm_panels_workspace_bytes(int64_t K, int64_t N, int64_t window_bytes, int64_t cap);
int64_t sddmm_panels_workspace_bytes(int64_t K, int64_t J, int64_t window_bytes, int64_t cap);
// row-split, serial strategy, one wavefront per rows_per_wave consecutive rows and 64 * vec columns
// (sgap_wave_rows.hip); skip = rows another kernel produces, or nullptr
hipError_t launch_wave_rows(const SpmmArgs& a, int vec, int rows_per_wave, int xcds, const RowSkip* skip,
                            hipStream_t s);
// zero the rows of C that receive atomic adds under a merge block of
// 2^merge_log2 positions, and the rows without entries; merge_log2 = -1: all rows
hipError_t launch_nnz_zero_rows(const SpmmArgs& a, int vec, int merge_log2, hipStream_t s);
// compute_units sizes the persistent grid; nnz_hint (-1 = unknown) caps it.
hipError_t launch_nnz_parallel(const SpmmArgs& a, int lc, int vec, int compute_units, int64_t nnz_hint, hipStream_t s);
hipError_t launch_nnz_serial(const SpmmArgs& a, int lc, int vec, const NnzPlan& plan, int compute_units,
                             int64_t nnz_hint, hipStream_t s);
// r = members per reducing sub-group (r = g: the whole group)
hipError_t launch_debug_group_reduce(const float* in, float* out, int g, int r, int lc, hipStream_t s);
// Sampled dense-dense product on A's pattern: a carries M, K, N = J, rowptr,
// colidx, vals and B = X2T (K x J); X1 is M x J; out has one value per stored
// entry.  g lanes per entry (per_lane = 0) or one lane per per_lane entries.
// row_cache lets the parallel strategy keep rows of X1 in registers where the shape allows.
hipError_t launch_sddmm(const SpmmArgs& a, const float* X1, float* out, int g, int per_lane, int vec, bool row_cache,
                        int compute_units, int64_t nnz_hint, hipStream_t stream);
// the same with the stored entries of rows of at least min_len entries produced
// window by window of X2T (sgap_panels.hip) and all others by the plain kernel;
// vec must be 4 and 32 <= J <= 256
hipError_t launch_sddmm_panels(const SpmmArgs& a, const float* X1, float* out, int g, int per_lane, int xcds,
                               int compute_units, int64_t nnz_hint, int32_t min_len, int64_t window_bytes,
                               void* workspace, int64_t cap, hipStream_t stream);
// the plain SDDMM kernel (no row cache) that leaves the entries of the rows described by `skip` alone
hipError_t launch_sddmm_skip(const SpmmArgs& a, const float* X1, float* out, int g, int per_lane, int compute_units,
                             int64_t nnz_hint, const RowSkip& skip, hipStream_t stream);
// MTTKRP on compressed sparse fibers: g lanes per slice (1 for the serial
// strategy), rows_per_slot slices per group (consecutive, or interleaved with
// the other groups' slices), lc chunk lanes of vec columns each.
hipError_t launch_mttkrp(int64_t I, int64_t K, int64_t L, int64_t J, const int32_t* fptr, const int32_t* fidx,
                         const int32_t* eptr, const int32_t* eidx, const float* vals, const float* X1,
                         const float* X2, float* Y, int g, int rows_per_slot, bool interleave, int lc, int vec,
                         int xcds, hipStream_t s);
hipError_t launch_debug_group_seg_reduce(const float* in, const int32_t* span, float* out, int g, int lc,
                                         hipStream_t s);
// MTTKRP with the stored entries as the unit of work (sgap_mttkrp_nnz.hip): g = lanes per segment group
// (parallel) or entries per lane (serial); Y must hold zeros.
hipError_t launch_mttkrp_nnz(const MttkrpArgs& a, int g, bool parallel, int lc, int vec, int compute_units,
                             int64_t nnz_hint, hipStream_t s);
// Rows grouped by a coarse key (sgap_reorder.hip): the permutation and the permuted copy of the matrix.
int64_t reorder_workspace_bytes(int64_t M);
hipError_t launch_reorder_rows(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colidx, const float* vals,
                               bool by_length, int32_t* perm, int32_t* rowptr_out, int32_t* colidx_out,
                               float* vals_out, void* workspace, int compute_units, hipStream_t s);

// Generic (g, lc, vec) -> template instance dispatch.  F is a functor with
//   template <int G, int LC, int VEC> void operator()() const
template <int G, int LC, typename F>
inline bool dispatch_vec(int vec, F&& f)
{
    switch (vec) {
        case 4: f.template operator()<G, LC, 4>(); return true;
        case 2: f.template operator()<G, LC, 2>(); return true;
        case 1: f.template operator()<G, LC, 1>(); return true;
        default: return false;
    }
}

template <int G, typename F>
inline bool dispatch_lc(int lc, int vec, F&& f)
{
    switch (lc) {
        case 1: if constexpr (G * 1 <= 64) return dispatch_vec<G, 1>(vec, f); break;
        case 2: if constexpr (G * 2 <= 64) return dispatch_vec<G, 2>(vec, f); break;
        case 4: if constexpr (G * 4 <= 64) return dispatch_vec<G, 4>(vec, f); break;
        case 8: if constexpr (G * 8 <= 64) return dispatch_vec<G, 8>(vec, f); break;
        case 16: if constexpr (G * 16 <= 64) return dispatch_vec<G, 16>(vec, f); break;
        case 32: if constexpr (G * 32 <= 64) return dispatch_vec<G, 32>(vec, f); break;
        case 64: if constexpr (G * 64 <= 64) return dispatch_vec<G, 64>(vec, f); break;
        default: break;
    }
    return false;
}

template <typename F>
inline bool dispatch_group(int g, int lc, int vec, F&& f)
{
    switch (g) {
        case 1: return dispatch_lc<1>(lc, vec, f);
        case 2: return dispatch_lc<2>(lc, vec, f);
        case 4: return dispatch_lc<4>(lc, vec, f);
        case 8: return dispatch_lc<8>(lc, vec, f);
        case 16: return dispatch_lc<16>(lc, vec, f);
        case 32: return dispatch_lc<32>(lc, vec, f);
        case 64: return dispatch_lc<64>(lc, vec, f);
        default: return false;
    }
}

}  // namespace sgap
