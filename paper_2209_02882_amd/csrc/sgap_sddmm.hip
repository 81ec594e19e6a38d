// Sampled dense-dense matrix product on the pattern of a CSR matrix
// (Section 2.1, the SDDMM form under Eq. 1):
//     out[p] = vals[p] * sum_{j<J} X1[row(p), j] * X2T[colidx[p], j]
// The paper's point in naming this operator next to SpMM is that the
// reduction is the same kind of object in both (Section 2.1: here it runs
// along the dense dimension j), so the same segment-group primitives serve:
//   parallel  G lanes share one stored entry, each takes every G-th chunk of
//             c columns of the two dense rows, the group tree-sums
//             (group_tree_sum, the library's atomicAddGroup) and its first
//             lane writes the entry: {<1 nnz, 1/g col>, g} in the notation of
//             Section 3.3 with the dense dimension split instead of a row.
//   serial    r = 1: a lane walks group_size consecutive stored entries by
//             itself, whole dot products in its own register.
// Every output has exactly one writer: no atomics, no zeroing.
//
// The unit of work is a stored entry, so the schedule is nnz-balanced by
// construction: tiles of 1024 entries are dealt to persistent workgroups
// (chunks of neighbouring tiles per die, see TileDeal), the rows of a tile's entries come from a bisection of rowptr
// for the tile's first entry and an LDS window of rowptr for the rest (the
// same pieces as the nnz-balanced SpMM kernels).
#include "sgap_common.hpp"
#include "sgap_lane_ops.hpp"
#include "sgap_nnz_common.hpp"

namespace sgap {

constexpr int kSddmmTile = 1024;   // stored entries per tile
constexpr int kSddmmDepth = 4;     // entries (parallel) or column chunks (serial) in flight per lane

struct SddmmArgs {
    SpmmArgs a;       // M, K, N = J, rowptr, colidx, vals; B = X2T; C unused
    const float* __restrict__ X1;
    float* __restrict__ out;
    RowSkip skip;     // entries of these rows are left alone (kernels instantiated with SKIP only)
};

template <int VEC>
__device__ __forceinline__ float dot_vec(const Vec<VEC>& x, const Vec<VEC>& y, float acc)
{
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc = __builtin_fmaf(x.v[i], y.v[i], acc);
    return acc;
}

// Copy the tile's columns and values into LDS and look up the row of every
// entry through the rowptr window (cut at row boundaries where long runs of
// empty rows overflow it).  row_lb = a row at or before the tile's first
// entry.  Block-uniform; the LDS arrays are ready on return.
// skip_len > 0: entries of rows of at least skip_len stored entries get the
// one's complement of their row (a negative number) instead.
__device__ __forceinline__ void stage_tile(const SpmmArgs& a, int32_t tile_start, int32_t tile_end, int32_t row_lb,
                                           int32_t* __restrict__ s_col, float* __restrict__ s_val,
                                           int32_t* __restrict__ s_row, int32_t* __restrict__ s_win,
                                           int32_t skip_len = 0)
{
    const int tid = threadIdx.x;
    const int cnt = tile_end - tile_start;
    __syncthreads();  // the previous tile is consumed
    for (int i = tid; i < cnt; i += kBlock) {
        s_col[i] = load_stream(a.colidx + tile_start + i);
        s_val[i] = load_stream(a.vals + tile_start + i);
    }
    for (int32_t base = tile_start; base < tile_end;) {
        __syncthreads();
        const RowWindow w = load_row_window(a, row_lb, base, tile_end - base, s_win);
        for (int i = tid; i < w.cnt; i += kBlock) {
            const int32_t wi = last_row_at_or_before(s_win, w.n_first, w.n_last, base + i);
            const bool skipped = skip_len > 0 && s_win[wi + 1] - s_win[wi] >= skip_len;
            s_row[base - tile_start + i] = skipped ? ~(row_lb + wi) : row_lb + wi;
        }
        row_lb += w.n_last;
        base += w.cnt;
    }
    __syncthreads();
}

// per_lane = 0: parallel strategy, G lanes per entry.  per_lane > 0 (G = 1):
// serial strategy, per_lane consecutive entries per lane.
// SKIP: leave the entries of the rows described by s.skip alone.
template <int G, int VEC, bool SKIP = false>
__global__ __launch_bounds__(kBlock) void sddmm_kernel(SddmmArgs s, int per_lane)
{
    __shared__ int32_t s_col[kSddmmTile];
    __shared__ float s_val[kSddmmTile];
    __shared__ int32_t s_row[kSddmmTile];
    __shared__ int32_t s_win[kWindowCap + 1];
    __shared__ int32_t s_tile_row[kTileRowBatch];
    constexpr int SLOTS = kBlock / G;

    const SpmmArgs& a = s.a;
    const int tid = threadIdx.x;
    const int slot = tid / G;
    const int member = tid % G;
    const int64_t J = a.N;
    const float* __restrict__ X2T = a.B;
    const int32_t nnz = a.rowptr[a.M];
    const int64_t tiles = ((int64_t)nnz + kSddmmTile - 1) / kSddmmTile;
    const TileDeal deal(tiles, blockIdx.x, gridDim.x);
    const int64_t my_tiles = deal.mine;
    if (my_tiles == 0) return;
    int32_t skip_len = 0;
    if constexpr (SKIP) skip_len = *s.skip.count <= s.skip.max_rows ? s.skip.min_len : 0;

    for (int64_t j0 = 0; j0 < my_tiles; j0 += kTileRowBatch) {
        find_tile_rows(a, deal, j0, kSddmmTile, s_tile_row);
        const int64_t j1 = j0 + kTileRowBatch < my_tiles ? j0 + kTileRowBatch : my_tiles;
        for (int64_t j = j0; j < j1; ++j) {
            const int64_t t = deal.tile(j);
            const int32_t tile_start = (int32_t)(t * kSddmmTile);
            const int32_t tile_end = nnz - tile_start < kSddmmTile ? nnz : tile_start + kSddmmTile;
            const int cnt = tile_end - tile_start;
            const int32_t row_lb = s_tile_row[j - j0];

            if constexpr (SKIP) {
                // a tile that lies inside one skipped row is not even staged (row_lb is the row of the tile's
                // first entry; the same two words for every lane, so the workgroup stays together)
                if (skip_len > 0 && a.rowptr[row_lb + 1] >= tile_end &&
                    a.rowptr[row_lb + 1] - a.rowptr[row_lb] >= skip_len)
                    continue;
            }
            stage_tile(a, tile_start, tile_end, row_lb, s_col, s_val, s_row, s_win, skip_len);

            if (per_lane == 0) {
                // U entries per group at a time, so that 2*U rows are in flight
                constexpr int U = kSddmmDepth;
                for (int e0 = 0; e0 < cnt; e0 += U * SLOTS) {  // same trip count in every lane
                    float acc[U];
                    const float* x1p[U];
                    const float* x2p[U];
                    bool ok[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int e = e0 + u * SLOTS + slot;
                        ok[u] = e < cnt;
                        if constexpr (SKIP) ok[u] = ok[u] && s_row[e] >= 0;
                        const int32_t row = ok[u] ? s_row[e] : 0;
                        const int32_t col = ok[u] ? s_col[e] : 0;
                        x1p[u] = s.X1 + (int64_t)row * J;
                        x2p[u] = X2T + (int64_t)col * J;
                        acc[u] = 0.0f;
                    }
                    for (int64_t c = (int64_t)member * VEC; c < J; c += (int64_t)G * VEC) {
                        Vec<VEC> x1[U], x2[U];
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            x1[u].zero();
                            x2[u].zero();
                            if (ok[u]) {
                                x1[u] = load_vec<VEC>(x1p[u] + c);
                                x2[u] = load_vec<VEC>(x2p[u] + c);
                            }
                        }
#pragma unroll
                        for (int u = 0; u < U; ++u) acc[u] = dot_vec<VEC>(x1[u], x2[u], acc[u]);
                    }
                    // members past the end of the dense rows contributed +0 (zero extension)
#pragma unroll
                    for (int u = 0; u < U; ++u) acc[u] = group_tree_sum<G, 1>(acc[u]);
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int e = e0 + u * SLOTS + slot;
                        if (member == 0 && ok[u]) s.out[tile_start + e] = s_val[e] * acc[u];
                    }
                }
            } else if constexpr (G == 1) {
                constexpr int U = kSddmmDepth;
                for (int i = 0; i < per_lane; ++i) {
                    for (int e = (tid * per_lane + i); e < cnt; e += kBlock * per_lane) {
                        if constexpr (SKIP) {
                            if (s_row[e] < 0) continue;
                        }
                        const float* __restrict__ x1p = s.X1 + (int64_t)s_row[e] * J;
                        const float* __restrict__ x2p = X2T + (int64_t)s_col[e] * J;
                        float acc = 0.0f;
                        int64_t c = 0;
                        for (; c + U * VEC <= J; c += U * VEC) {
                            Vec<VEC> x1[U], x2[U];
#pragma unroll
                            for (int u = 0; u < U; ++u) {
                                x1[u] = load_vec<VEC>(x1p + c + u * VEC);
                                x2[u] = load_vec<VEC>(x2p + c + u * VEC);
                            }
#pragma unroll
                            for (int u = 0; u < U; ++u) acc = dot_vec<VEC>(x1[u], x2[u], acc);
                        }
                        for (; c < J; c += VEC) acc = dot_vec<VEC>(load_vec<VEC>(x1p + c), load_vec<VEC>(x2p + c), acc);
                        s.out[tile_start + e] = s_val[e] * acc;
                    }
                }
            }
        }
    }
}

// Parallel strategy when the G lanes of a group cover a dense row in S <= 4
// steps of 4 columns each (J <= S*G*4, 16-byte aligned operands).
// A group takes its stored entries in batches of U CONSECUTIVE ones, which
// mostly belong to one row of A, and keeps that row's chunk of X1 in
// registers: a row of X1 is loaded when the row changes, not once per entry,
// which takes up to half of the volume off the vector memory path.  The
// batches of a round are dealt to the groups in order, so that the workgroup
// as a whole still moves through neighbouring entries, whose rows of X2T tend
// to be neighbours or the same (L1 hits).  The loads of a batch (rows of X2T,
// and rows of X1 where the row changes inside the batch) are issued together.
template <int G, int S>
__global__ __launch_bounds__(kBlock) void sddmm_rowcache_kernel(SddmmArgs s)
{
    constexpr int VEC = 4;
    constexpr int SLOTS = kBlock / G;
    constexpr int EPS = kSddmmTile / SLOTS;  // entries per group and tile
    constexpr int U = 8 / S < EPS ? 8 / S : EPS;  // entries per batch: U*S <= 8 loads per operand in flight
    __shared__ int32_t s_col[kSddmmTile];
    __shared__ float s_val[kSddmmTile];
    __shared__ int32_t s_row[kSddmmTile];
    __shared__ int32_t s_win[kWindowCap + 1];
    __shared__ int32_t s_tile_row[kTileRowBatch];

    const SpmmArgs& a = s.a;
    const int tid = threadIdx.x;
    const int slot = tid / G;
    const int member = tid % G;
    const int64_t J = a.N;
    const float* __restrict__ X2T = a.B;
    const int32_t nnz = a.rowptr[a.M];
    const int64_t tiles = ((int64_t)nnz + kSddmmTile - 1) / kSddmmTile;
    const TileDeal deal(tiles, blockIdx.x, gridDim.x);
    const int64_t my_tiles = deal.mine;
    if (my_tiles == 0) return;
    // this lane's columns: (st*G + member)*4, st < S
    bool c_ok[S];
#pragma unroll
    for (int st = 0; st < S; ++st) c_ok[st] = (int64_t)(st * G + member) * VEC < J;

    for (int64_t j0 = 0; j0 < my_tiles; j0 += kTileRowBatch) {
        find_tile_rows(a, deal, j0, kSddmmTile, s_tile_row);
        const int64_t j1 = j0 + kTileRowBatch < my_tiles ? j0 + kTileRowBatch : my_tiles;
        for (int64_t j = j0; j < j1; ++j) {
            const int64_t t = deal.tile(j);
            const int32_t tile_start = (int32_t)(t * kSddmmTile);
            const int32_t tile_end = nnz - tile_start < kSddmmTile ? nnz : tile_start + kSddmmTile;
            const int cnt = tile_end - tile_start;
            const int32_t row_lb = s_tile_row[j - j0];

            stage_tile(a, tile_start, tile_end, row_lb, s_col, s_val, s_row, s_win);

            int32_t cur_row = -1;
            Vec<VEC> x1c[S];  // the chunk of X1[cur_row] this lane owns
#pragma unroll
            for (int st = 0; st < S; ++st) x1c[st].zero();
            for (int i0 = 0; i0 < EPS; i0 += U) {  // same trip count in every lane
                int32_t row[U], col[U];
                bool ok[U], fresh[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int e = (i0 / U * SLOTS + slot) * U + u;
                    ok[u] = e < cnt;
                    row[u] = ok[u] ? s_row[e] : (u ? row[u - 1] : cur_row);
                    col[u] = ok[u] ? s_col[e] : 0;
                    fresh[u] = ok[u] && row[u] != (u ? row[u - 1] : cur_row);
                }
                Vec<VEC> x1[U][S], x2[U][S];
#pragma unroll
                for (int u = 0; u < U; ++u) {
#pragma unroll
                    for (int st = 0; st < S; ++st) {
                        const int64_t c = (int64_t)(st * G + member) * VEC;
                        x2[u][st].zero();
                        x1[u][st].zero();
                        if (ok[u] && c_ok[st]) x2[u][st] = load_vec<VEC>(X2T + (int64_t)col[u] * J + c);
                        if (fresh[u] && c_ok[st]) x1[u][st] = load_vec<VEC>(s.X1 + (int64_t)row[u] * J + c);
                    }
                }
                float acc[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    acc[u] = 0.0f;
#pragma unroll
                    for (int st = 0; st < S; ++st) {
                        if (fresh[u]) x1c[st] = x1[u][st];
                        acc[u] = dot_vec<VEC>(x1c[st], x2[u][st], acc[u]);
                    }
                }
                cur_row = row[U - 1];
#pragma unroll
                for (int u = 0; u < U; ++u) acc[u] = group_tree_sum<G, 1>(acc[u]);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int e = (i0 / U * SLOTS + slot) * U + u;
                    if (member == 0 && ok[u]) s_val[e] *= acc[u];  // this group is the entry's only reader
                }
            }
            __syncthreads();
            for (int i = tid; i < cnt; i += kBlock) s.out[tile_start + i] = s_val[i];
        }
    }
}

namespace {

template <int G, int S>
void launch_rowcache(const SddmmArgs& s, int compute_units, int64_t nnz_hint, hipStream_t stream)
{
    static const int per_cu = resident_per_cu(sddmm_rowcache_kernel<G, S>, 0);
    const int grid = persistent_grid(per_cu, compute_units, nnz_hint, kSddmmTile);
    hipLaunchKernelGGL((sddmm_rowcache_kernel<G, S>), dim3(grid), dim3(kBlock), 0, stream, s);
}

// steps of G*4 columns that cover J: 1, 2 or 4 pick the row-cache kernel, 0 = more than 4
template <int G>
bool try_rowcache(const SddmmArgs& s, int64_t J, int compute_units, int64_t nnz_hint, hipStream_t stream)
{
    const int64_t steps = (J + G * 4 - 1) / (G * 4);
    if (steps <= 1) launch_rowcache<G, 1>(s, compute_units, nnz_hint, stream);
    else if (steps <= 2) launch_rowcache<G, 2>(s, compute_units, nnz_hint, stream);
    else if (steps <= 4) launch_rowcache<G, 4>(s, compute_units, nnz_hint, stream);
    else return false;
    return true;
}

template <int G, int VEC>
void launch_one(const SddmmArgs& s, int per_lane, int compute_units, int64_t nnz_hint, hipStream_t stream)
{
    static const int per_cu = resident_per_cu(sddmm_kernel<G, VEC>, 0);
    const int grid = persistent_grid(per_cu, compute_units, nnz_hint, kSddmmTile);
    hipLaunchKernelGGL((sddmm_kernel<G, VEC>), dim3(grid), dim3(kBlock), 0, stream, s, per_lane);
}

template <int G>
void launch_skip(const SddmmArgs& s, int per_lane, int compute_units, int64_t nnz_hint, hipStream_t stream)
{
    static const int per_cu = resident_per_cu(sddmm_kernel<G, 4, true>, 0);
    const int grid = persistent_grid(per_cu, compute_units, nnz_hint, kSddmmTile);
    hipLaunchKernelGGL((sddmm_kernel<G, 4, true>), dim3(grid), dim3(kBlock), 0, stream, s, per_lane);
}

template <int G>
bool launch_vec(const SddmmArgs& s, int vec, int per_lane, int compute_units, int64_t nnz_hint, hipStream_t stream)
{
    switch (vec) {
        case 4: launch_one<G, 4>(s, per_lane, compute_units, nnz_hint, stream); return true;
        case 2: launch_one<G, 2>(s, per_lane, compute_units, nnz_hint, stream); return true;
        case 1: launch_one<G, 1>(s, per_lane, compute_units, nnz_hint, stream); return true;
        default: return false;
    }
}

}  // namespace

// a: M, K, N = J, rowptr, colidx, vals, B = X2T (C unused).  g = lanes per
// stored entry (parallel strategy, per_lane = 0) or 1 with per_lane = entries
// per lane (serial strategy).  vec = columns per lane and load (4, 2 or 1;
// J % vec == 0 and matching alignment of X1 and X2T).
// row_cache: let the parallel strategy keep rows of X1 in registers where the
// shape allows it.
hipError_t launch_sddmm(const SpmmArgs& a, const float* X1, float* out, int g, int per_lane, int vec, bool row_cache,
                        int compute_units, int64_t nnz_hint, hipStream_t stream)
{
    SddmmArgs s;
    s.a = a;
    s.X1 = X1;
    s.out = out;
    s.skip = RowSkip{nullptr, 0, 0};
    bool ok = false;
    if (per_lane > 0) {
        ok = launch_vec<1>(s, vec, per_lane, compute_units, nnz_hint, stream);
    } else if (vec == 4 && row_cache && a.N > 0) {
        switch (g) {
            case 1: ok = try_rowcache<1>(s, a.N, compute_units, nnz_hint, stream); break;
            case 2: ok = try_rowcache<2>(s, a.N, compute_units, nnz_hint, stream); break;
            case 4: ok = try_rowcache<4>(s, a.N, compute_units, nnz_hint, stream); break;
            case 8: ok = try_rowcache<8>(s, a.N, compute_units, nnz_hint, stream); break;
            case 16: ok = try_rowcache<16>(s, a.N, compute_units, nnz_hint, stream); break;
            case 32: ok = try_rowcache<32>(s, a.N, compute_units, nnz_hint, stream); break;
            case 64: ok = try_rowcache<64>(s, a.N, compute_units, nnz_hint, stream); break;
            default: break;
        }
        if (!ok) return launch_sddmm(a, X1, out, g, per_lane, vec, false, compute_units, nnz_hint, stream);
    } else {
        switch (g) {
            case 1: ok = launch_vec<1>(s, vec, 0, compute_units, nnz_hint, stream); break;
            case 2: ok = launch_vec<2>(s, vec, 0, compute_units, nnz_hint, stream); break;
            case 4: ok = launch_vec<4>(s, vec, 0, compute_units, nnz_hint, stream); break;
            case 8: ok = launch_vec<8>(s, vec, 0, compute_units, nnz_hint, stream); break;
            case 16: ok = launch_vec<16>(s, vec, 0, compute_units, nnz_hint, stream); break;
            case 32: ok = launch_vec<32>(s, vec, 0, compute_units, nnz_hint, stream); break;
            case 64: ok = launch_vec<64>(s, vec, 0, compute_units, nnz_hint, stream); break;
            default: break;
        }
    }
    if (!ok) return hipErrorInvalidValue;
    return hipGetLastError();
}

// The plain kernel (16-byte loads: J % 4 == 0, aligned operands) with the
// entries of the rows described by `skip` left alone.
hipError_t launch_sddmm_skip(const SpmmArgs& a, const float* X1, float* out, int g, int per_lane, int compute_units,
                             int64_t nnz_hint, const RowSkip& skip, hipStream_t stream)
{
    SddmmArgs s;
    s.a = a;
    s.X1 = X1;
    s.out = out;
    s.skip = skip;
    switch (per_lane > 0 ? 1 : g) {
        case 1: launch_skip<1>(s, per_lane, compute_units, nnz_hint, stream); break;
        case 2: launch_skip<2>(s, per_lane, compute_units, nnz_hint, stream); break;
        case 4: launch_skip<4>(s, per_lane, compute_units, nnz_hint, stream); break;
        case 8: launch_skip<8>(s, per_lane, compute_units, nnz_hint, stream); break;
        case 16: launch_skip<16>(s, per_lane, compute_units, nnz_hint, stream); break;
        case 32: launch_skip<32>(s, per_lane, compute_units, nnz_hint, stream); break;
        case 64: launch_skip<64>(s, per_lane, compute_units, nnz_hint, stream); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sgap
