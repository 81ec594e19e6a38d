// MTTKRP on compressed sparse fibers (Section 2.1, the first of the forms
// listed under Eq. 1):   Y[i,j] = sum_{k,l} A[i,k,l] * X1[k,j] * X2[l,j].
//
// The operator holds two reductions of the SpMM kind, one inside the other
// (Section 2.1: the result of the first is the input of the second):
//   first level,  over the entries of a fiber (i,k):  t[j]  = sum_l A[i,k,l] * X2[l,j]
//   second level, over the fibers of a slice i:        Y[i,j] = sum_k X1[k,j] * t[j]
// Both are row-split reductions: a slice is produced by exactly one group, so
// results are written with plain stores and empty slices are written as zeros.
//
//   parallel  G lanes per slice ({<1/g row, c col>, r} with g = r = G, Section
//             6.2): member m takes the slice's fibers m, m+G, ...; each member
//             runs the first-level reduction of its fibers serially and adds
//             X1[k,:] * t into its own accumulator; because the second level
//             is linear in t the group tree-sums once per slice, and member 0
//             stores.
//   serial    one lane per slice and column chunk, `group_size` consecutive
//             slices per lane ({<g row, c col>, 1}, Section 6.1).
// Lane layout:  thread = (slot*G + member)*LC + chunk over the workgroup; the
// LC chunk lanes of a member hold neighbouring column chunks of VEC columns.
//
// Compressed fibers put three dependent loads (slice pointer, fiber, entries)
// before the first row of X2 can be asked for.  A workgroup therefore copies
// the three levels of its block of slices into LDS with coalesced loads, three
// memory round trips per block, and its lanes then walk fibers and entries out
// of LDS: the vector memory path carries the gathered rows of X1 and X2 and
// little else.  A block too large for the LDS copies is worked through straight
// from memory, fiber by fiber.
#include "sgap_common.hpp"
#include "sgap_gather.hpp"
#include "sgap_lane_ops.hpp"

namespace sgap {

constexpr int kMttkrpDepth = 4;  // gathered rows of X2 in flight per lane when entries come straight from memory

// LDS copies of a block of slices: its slice pointers, its fibers (second index
// and entry pointer) and its entries.  A block that does not fit is worked
// through straight from memory.
constexpr int kMtRows = 256;     // slices per block at most (+1 pointers)
constexpr int kMtFibers = 512;   // fibers (+1 pointers)
constexpr int kMtEntries = 2048; // (third index, value) pairs: 16 KB

// value of chunk lane `src` (0 <= src < LC) of this lane's aligned run of LC lanes
template <int LC>
__device__ __forceinline__ int32_t from_chunk_lane(int32_t v, int src)
{
    if constexpr (LC == 1) return v;
    else return __shfl(v, src, LC);
}

// One member's share of a slice, fibers f_begin + member, + G, ... < f_end, with
// every level read from memory: the next fiber's (second index, entry range) is
// asked for one fiber ahead, the fiber's row of X1 travels with its first
// entries, and the LC chunk lanes load LC entries with one coalesced load and
// hand the (index, value) pairs round through the LDS crossbar.
template <int G, int LC, int VEC, bool OFF32>
__device__ __forceinline__ void mttkrp_slice_direct(const MttkrpArgs& a, Vec<VEC>& acc, int32_t f_begin, int32_t f_end,
                                                    int member, int chunk, int64_t k, bool k_ok,
                                                    const BRow<OFF32>& x2row)
{
    constexpr int D = kMttkrpDepth;
    int32_t f = f_begin + member;
    int32_t next_k = 0, next_begin = 0, next_end = 0;
    if (f < f_end) {
        next_k = a.fidx[f];
        next_begin = a.eptr[f];
        next_end = a.eptr[f + 1];
    }
    for (; f < f_end; f += G) {
        const int32_t fiber_k = next_k, e_begin = next_begin, e_end = next_end;
        if (f + G < f_end) {
            next_k = a.fidx[f + G];
            next_begin = a.eptr[f + G];
            next_end = a.eptr[f + G + 1];
        }
        Vec<VEC> x1;
        x1.zero();
        if (k_ok) x1 = load_vec<VEC>(a.X1 + (int64_t)fiber_k * a.J + k);
        Vec<VEC> t;
        t.zero();
        for (int32_t base = e_begin; base < e_end; base += LC) {
            // the LC chunk lanes of this member are all here: one entry each
            int32_t my_idx = 0, my_val = 0;
            if (base + chunk < e_end) {
                my_idx = load_stream(a.eidx + base + chunk);
                my_val = __float_as_int(load_stream(a.vals + base + chunk));
            }
            const int cnt = e_end - base < LC ? e_end - base : LC;
            for (int j = 0; j < cnt; j += D) {
                int32_t idx[D];
                float val[D];
                Vec<VEC> b[D];
#pragma unroll
                for (int u = 0; u < D; ++u) {
                    // lanes past the end of the fiber hold (0, +0); past LC the source wraps and is masked
                    idx[u] = from_chunk_lane<LC>(my_idx, (j + u) % LC);
                    val[u] = __int_as_float(from_chunk_lane<LC>(my_val, (j + u) % LC));
                    if (j + u >= cnt) val[u] = 0.0f;
                }
#pragma unroll
                for (int u = 0; u < D; ++u) {
                    b[u].zero();
                    if (k_ok && j + u < cnt) b[u] = load_vec<VEC>(x2row.at(idx[u]));
                }
#pragma unroll
                for (int u = 0; u < D; ++u) t.fma(val[u], b[u]);
            }
        }
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc.v[i] = __builtin_fmaf(x1.v[i], t.v[i], acc.v[i]);
    }
}

template <int G, int LC, int VEC, bool OFF32>
__global__ __launch_bounds__(kBlock) void mttkrp_kernel(MttkrpArgs a, int rows_per_slot, int interleave,
                                                        int64_t row_blocks, int64_t blocks_per_xcd, int xcds)
{
    __shared__ StagedEntry s_A[kMtEntries];
    __shared__ int32_t s_fk[kMtFibers];
    __shared__ int32_t s_ep[kMtFibers + 1];
    __shared__ int32_t s_fp[kMtRows + 1];
    constexpr int SPAN = G * LC;
    constexpr int SLOTS = kBlock / SPAN;
    const int slot = threadIdx.x / SPAN;
    const int member = (threadIdx.x / LC) % G;
    const int chunk = threadIdx.x % LC;

    // workgroup b runs on die b % xcds: every die gets one contiguous run of row blocks
    const int64_t row_block = (int64_t)(blockIdx.x % xcds) * blocks_per_xcd + blockIdx.x / xcds;
    if (row_block >= row_blocks) return;  // the whole workgroup
    const int64_t rows_per_block = (int64_t)SLOTS * rows_per_slot;
    const int64_t row_first = row_block * rows_per_block;
    const int64_t row_last = row_first + rows_per_block < a.I ? row_first + rows_per_block : a.I;
    const int block_rows = (int)(row_last - row_first);

    // Bring the block's three levels into LDS, each with coalesced loads of the
    // whole workgroup: three memory round trips per block instead of three per
    // fiber.  Every test below reads the same LDS words in all lanes, so the
    // workgroup takes the same way through the barriers.
    bool staged = false;
    int32_t f0 = 0, e0 = 0;
    if (rows_per_block <= kMtRows) {
        for (int i = threadIdx.x; i <= block_rows; i += kBlock) s_fp[i] = a.fptr[row_first + i];
        __syncthreads();
        f0 = s_fp[0];
        const int32_t fibers = s_fp[block_rows] - f0;
        if (fibers >= 0 && fibers <= kMtFibers) {
            for (int i = threadIdx.x; i <= fibers; i += kBlock) {
                s_ep[i] = a.eptr[f0 + i];
                if (i < fibers) s_fk[i] = a.fidx[f0 + i];
            }
            __syncthreads();
            e0 = s_ep[0];
            const int32_t entries = s_ep[fibers] - e0;
            if (entries >= 0 && entries <= kMtEntries) {
                for (int i = threadIdx.x; i < entries; i += kBlock) {
                    StagedEntry e;
                    e.col = load_stream(a.eidx + e0 + i);
                    e.val = load_stream(a.vals + e0 + i);
                    s_A[i] = e;
                }
                __syncthreads();
                staged = true;
            }
        }
    }

    for (int64_t k0 = 0; k0 < a.J; k0 += (int64_t)LC * VEC) {
        const int64_t k = k0 + (int64_t)chunk * VEC;
        const bool k_ok = k < a.J;
        const BRow<OFF32> x2row(a.X2, a.J, k_ok ? k : 0);
        const GlobalRows<VEC, OFF32> x2rows(a.X2, a.J, k_ok ? k : 0);
        for (int r = 0; r < rows_per_slot; ++r) {
            // the lanes of a slot share `row`, so whole slots leave together
            const int64_t row = row_first + (interleave ? slot + (int64_t)r * SLOTS : (int64_t)slot * rows_per_slot + r);
            if (row >= row_last) break;
            Vec<VEC> acc;
            acc.zero();
            if (staged) {
                const int32_t f_end = s_fp[row - row_first + 1] - f0;
                for (int32_t f = s_fp[row - row_first] - f0 + member; f < f_end; f += G) {
                    // the fiber's row of X1 is in flight while its entries are multiplied out
                    Vec<VEC> x1, t;
                    x1.zero();
                    t.zero();
                    if (k_ok) {
                        x1 = load_vec<VEC>(a.X1 + (int64_t)s_fk[f] * a.J + k);
                        const uint32_t q0 = (uint32_t)(s_ep[f] - e0), q1 = (uint32_t)(s_ep[f + 1] - e0);
                        if (q0 < q1) gather_fma<VEC, 1>(t, s_A, q0, q1, x2rows);
                    }
#pragma unroll
                    for (int i = 0; i < VEC; ++i) acc.v[i] = __builtin_fmaf(x1.v[i], t.v[i], acc.v[i]);
                }
            } else {
                mttkrp_slice_direct<G, LC, VEC, OFF32>(a, acc, a.fptr[row], a.fptr[row + 1], member, chunk, k, k_ok,
                                                       x2row);
            }
            // members without fibers contributed +0; the lanes of a slot meet here
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc.v[i] = group_tree_sum<G, LC>(acc.v[i]);
            if (member == 0 && k_ok) store_vec_stream<VEC>(a.Y + row * a.J + k, acc);
        }
    }
}

namespace {

struct LaunchMttkrp {
    const MttkrpArgs& a;
    int rows_per_slot, interleave, xcds;
    bool off32;
    hipStream_t s;
    template <int G, int LC, int VEC>
    void operator()() const
    {
        constexpr int slots = kBlock / (G * LC);
        const int64_t rows_per_block = (int64_t)slots * rows_per_slot;
        const int64_t row_blocks = (a.I + rows_per_block - 1) / rows_per_block;
        const int64_t blocks_per_xcd = (row_blocks + xcds - 1) / xcds;
        const unsigned grid = (unsigned)(blocks_per_xcd * xcds);
        if (off32)
            hipLaunchKernelGGL((mttkrp_kernel<G, LC, VEC, true>), dim3(grid), dim3(kBlock), 0, s, a, rows_per_slot,
                               interleave, row_blocks, blocks_per_xcd, xcds);
        else
            hipLaunchKernelGGL((mttkrp_kernel<G, LC, VEC, false>), dim3(grid), dim3(kBlock), 0, s, a, rows_per_slot,
                               interleave, row_blocks, blocks_per_xcd, xcds);
    }
};

}  // namespace

// g = lanes per slice (1 for the serial strategy), rows_per_slot = slices a
// group works through (consecutive ones, or every slots-th slice of the block
// when `interleave` is set), lc = chunk lanes, vec = columns per lane.
hipError_t launch_mttkrp(int64_t I, int64_t K, int64_t L, int64_t J, const int32_t* fptr, const int32_t* fidx,
                         const int32_t* eptr, const int32_t* eidx, const float* vals, const float* X1,
                         const float* X2, float* Y, int g, int rows_per_slot, bool interleave, int lc, int vec,
                         int xcds, hipStream_t s)
{
    MttkrpArgs a{I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2, Y};
    // every byte offset into X2 fits 32 bits and both factors of it fit 24 bits
    const bool off32 = L <= (1 << 24) && J * 4 < (1 << 24) && L * J * 4 <= 0xffffffffLL;
    const int64_t rows_per_block = (int64_t)(kBlock / (g * lc)) * rows_per_slot;
    if ((I + rows_per_block - 1) / rows_per_block + xcds > 0x7ffffff0LL) return hipErrorInvalidValue;
    LaunchMttkrp f{a, rows_per_slot, interleave ? 1 : 0, xcds, off32, s};
    if (!dispatch_group(g, lc, vec, f)) return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace sgap
