// MTTKRP on compressed sparse fibers with the stored entries as the unit of work (the nnz-balanced
// schedule of Section 6 carried over to the operator of Section 2.1 that holds two nested reductions,
// the second fed by the first):
//     t[f,:]  = sum over the entries (l, v) of fiber f of  v * X2[l,:]           (first reduction)
//     Y[i,:]  = sum over the fibers f of slice i of        X1[fidx[f],:] * t[f,:]  (second reduction)
// Stored entries are cut into tiles of kMtTile positions, whatever slices and fibers they fall in, so a
// tensor with a few huge slices keeps the whole chip busy.
//   parallel  {<1 nnz, c col>, r}, r = G: a lane multiplies one entry by its chunk of the row of X2; the G
//             members of a group run a segmented sum keyed by fiber; the first lane of every fiber run
//             multiplies by its chunk of the row of X1; a second segmented sum, keyed by slice, runs over
//             those products (the other lanes pass +0); the first lane of every slice run adds into Y.
//   serial    {<g nnz, c col>, 1}: a lane walks G consecutive entries, closes a fiber's sum into the
//             slice's sum where the fiber (or its share) ends, and adds the slice's sum into Y where the
//             slice (or its share) ends: the conditional flush, twice.
// Lane layout as everywhere: thread = (slot*G + member)*LC + chunk.  Several groups may hold parts of one
// slice, so sums are ADDED into Y (the "Atomics" output strategy of Section 6.2) and Y is set to zero
// beforehand.  Where the accumulators fit (tile mode of the SpMM kernels' merge rule: one slot per aligned
// block of G positions, for the slice that starts in it and goes on past it, and one for the slice that
// entered the tile from the left) the runs of a slice inside a tile are first combined in LDS and leave
// with one atomic row per slice and tile; else every run adds into Y by itself.  Fiber and slice of an entry come from bisections of the two pointer arrays inside
// windows of 1,025 pointers kept in LDS (the tile's first fiber and slice are found by the workgroup
// together); an entry whose fiber or slice lies beyond a window (long runs of fibers or slices without
// entries) bisects the arrays themselves.
#include "sgap_common.hpp"
#include "sgap_lane_ops.hpp"
#include "sgap_nnz_common.hpp"

namespace sgap {

constexpr int kMtTile = 1024;  // stored entries per tile
constexpr int kMtWin = 1024;   // pointers per window (+1)
constexpr int kMtFirstFiber = 1, kMtFirstSlice = 2, kMtValid = 4;

struct __align__(16) MtRecord {
    int32_t l;    // third index: row of X2
    float val;
    int32_t k;    // second index of the entry's fiber: row of X1
    int32_t i;    // slice: row of Y
};

// Entries that follow this lane's entry inside its group before the next run starts (at most `room`).
// starts = ballot of "my entry starts a run" (the LC lanes of an entry agree).
template <int LC>
__device__ __forceinline__ int run_span(unsigned long long starts, int entry_lane, int room)
{
    const int sh = (entry_lane + 1) * LC;
    const unsigned long long m = sh < kWave ? starts >> sh : 0ull;
    const int following = m ? (__ffsll((long long)m) - 1) / LC : kWave;
    return following < room ? following : room;
}

template <int G, int LC, int VEC, bool PAR, bool MERGE>
__global__ __launch_bounds__(kBlock) void mttkrp_nnz_kernel(MttkrpArgs a, int group, int log2_group)
{
    extern __shared__ __align__(16) unsigned char s_raw[];
    __shared__ MtRecord s_rec[kMtTile];
    __shared__ uint8_t s_flag[kMtTile];
    __shared__ uint16_t s_slot[kMtTile];
    __shared__ int32_t s_ewin[kMtWin + 1];
    __shared__ int32_t s_fwin[kMtWin + 1];
    const int tid = threadIdx.x;
    const int32_t I = (int32_t)a.I;
    const int32_t F = a.fptr[a.I];
    const int32_t E = F > 0 ? a.eptr[F] : 0;
    const int64_t tiles = ((int64_t)E + kMtTile - 1) / kMtTile;
    SpmmArgs out;  // what write_out and merge_write_out need
    out.N = a.J;
    out.C = a.Y;
    MergeBuf mb;
    mb.nslots = (kMtTile >> log2_group) + 1;
    mb.width = LC * VEC;
    mb.accum = reinterpret_cast<float*>(s_raw);
    mb.slot_row = reinterpret_cast<int32_t*>(mb.accum + (MERGE ? mb.nslots * mb.width : 0));
    mb.slot_atomic = mb.slot_row + mb.nslots;
    if constexpr (MERGE) merge_reset(mb);  // made visible by the barriers below

    for (int64_t t = blockIdx.x; t < tiles; t += gridDim.x) {
        const int32_t tile_start = (int32_t)(t * kMtTile);
        const int32_t cnt = E - tile_start < kMtTile ? E - tile_start : kMtTile;
        // the fiber of the tile's first entry and that fiber's slice
        const int32_t f0 = find_row_cooperative(a.eptr, 0, F - 1, tile_start);
        const int32_t i0 = find_row_cooperative(a.fptr, 0, I - 1, f0);
        __syncthreads();  // the previous tile's records and windows are no longer read
        for (int w = tid; w <= kMtWin; w += kBlock) {
            const int64_t f = (int64_t)f0 + w, i = (int64_t)i0 + w;
            s_ewin[w] = a.eptr[f <= F ? f : F];
            s_fwin[w] = a.fptr[i <= I ? i : I];
        }
        __syncthreads();
        for (int q = tid; q < kMtTile; q += kBlock) {
            MtRecord r;
            r.l = 0; r.val = 0.0f; r.k = 0; r.i = 0;
            int flag = 0, slot = 0;
            if (q < cnt) {
                const int32_t p = tile_start + q;
                int32_t f, e_begin;
                if (s_ewin[kMtWin] > p) {
                    const int32_t w = first_above(s_ewin, kMtWin + 1, p) - 1;  // last window fiber starting at or before p
                    f = f0 + w;
                    e_begin = s_ewin[w];
                } else {
                    f = last_row_at_or_before(a.eptr, f0 + kMtWin, F - 1, p);
                    e_begin = a.eptr[f];
                }
                int32_t i, f_begin;
                if (s_fwin[kMtWin] > f) {
                    const int32_t w = first_above(s_fwin, kMtWin + 1, f) - 1;
                    i = i0 + w;
                    f_begin = s_fwin[w];
                } else {
                    i = last_row_at_or_before(a.fptr, i0 + kMtWin, I - 1, f);
                    f_begin = a.fptr[i];
                }
                // the slice's first entry is where its first fiber's entries start (fibers without entries in front
                // of it share that position)
                const int32_t s_begin =
                    f_begin >= f0 && f_begin - f0 <= kMtWin ? s_ewin[f_begin - f0] : a.eptr[f_begin];
                r.l = a.eidx[p];
                r.val = a.vals[p];
                r.k = a.fidx[f];
                r.i = i;
                flag = kMtValid | (p == e_begin ? kMtFirstFiber : 0) | (p == s_begin ? kMtFirstSlice : 0);
                slot = s_begin < tile_start ? mb.nslots - 1 : (s_begin - tile_start) >> log2_group;
            }
            s_rec[q] = r;
            s_flag[q] = (uint8_t)flag;
            s_slot[q] = (uint16_t)slot;
        }
        __syncthreads();

        if constexpr (PAR) {
            constexpr int ENTRIES_PER_WAVE = kWave / LC;
            constexpr int ENTRIES_PER_STEP = ENTRIES_PER_WAVE * kWavesPerBlock;
            constexpr int STEPS = kMtTile / ENTRIES_PER_STEP;
            const int lane = tid & (kWave - 1);
            const int wave = tid / kWave;
            const int entry_lane = lane / LC;  // = slot*G + member
            const int member = entry_lane % G;
            const int chunk = lane % LC;
            for (int64_t k0 = 0; k0 < a.J; k0 += (int64_t)LC * VEC) {
                const int64_t k = k0 + (int64_t)chunk * VEC;
                const bool k_ok = k < a.J;
                for (int step = 0; step < STEPS; ++step) {
                    const int q = (step * kWavesPerBlock + wave) * ENTRIES_PER_WAVE + entry_lane;
                    if ((step * kWavesPerBlock + wave) * ENTRIES_PER_WAVE >= cnt) break;  // the whole wavefront
                    const MtRecord r = s_rec[q];
                    const int fl = s_flag[q];
                    const bool valid = (fl & kMtValid) != 0;
                    Vec<VEC> x;
                    x.zero();
                    if (valid && k_ok) {
                        x = load_vec<VEC>(a.X2 + (int64_t)r.l * a.J + k);
#pragma unroll
                        for (int v = 0; v < VEC; ++v) x.v[v] *= r.val;
                    }
                    // a run starts at member 0, at a fiber's (slice's) first entry, and at every position past the end
                    const bool start_f = !valid || member == 0 || (fl & kMtFirstFiber);
                    const bool start_s = !valid || member == 0 || (fl & kMtFirstSlice);
                    const int span_f = run_span<LC>(__ballot(start_f), entry_lane, G - 1 - member);
                    const int span_s = run_span<LC>(__ballot(start_s), entry_lane, G - 1 - member);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) x.v[v] = group_seg_sum<G, LC>(x.v[v], span_f);
                    // the second reduction is fed by the first: fiber runs' sums times the fiber's row of X1
                    Vec<VEC> y;
                    y.zero();
                    if (valid && start_f && k_ok) {
                        const Vec<VEC> x1 = load_vec<VEC>(a.X1 + (int64_t)r.k * a.J + k);
#pragma unroll
                        for (int v = 0; v < VEC; ++v) y.v[v] = x1.v[v] * x.v[v];
                    }
#pragma unroll
                    for (int v = 0; v < VEC; ++v) y.v[v] = group_seg_sum<G, LC>(y.v[v], span_s);
                    if constexpr (MERGE) {
                        // A slice that lies inside the group (it starts at this lane and the next slice starts
                        // before the group ends) has no other writer: plain store.  Every other run goes to the
                        // slot of its slice; the slot's owner is the run that holds the slice's first entry
                        // inside the tile.
                        const unsigned long long firsts = __ballot(valid && (fl & kMtFirstSlice));
                        const bool inside = (fl & kMtFirstSlice) && run_span<LC>(firsts, entry_lane, kWave) < G - 1 - member;
                        if (valid && start_s && k_ok) {
                            if (inside)
                                write_out<LC, VEC>(out, r.i, k, true, y);
                            else
                                merge_add<VEC, false>(mb, s_slot[q], chunk * VEC, y,
                                                      chunk == 0 && ((fl & kMtFirstSlice) || q == 0), r.i, true);
                        }
                    } else {
                        if (valid && start_s && k_ok) write_out<LC, VEC>(out, r.i, k, false, y);
                    }
                }
                if constexpr (MERGE) {
                    __syncthreads();  // all sums of this pass are in LDS
                    merge_write_out<LC, VEC>(out, mb, k, k_ok);
                    __syncthreads();  // slots are clear again
                }
            }
        } else {
            constexpr int D = 4;  // rows of X2 in flight per lane
            constexpr int ENTRY_LANES = kBlock / LC;
            const int entry_lane = tid / LC;
            const int chunk = tid % LC;
            for (int64_t k0 = 0; k0 < a.J; k0 += (int64_t)LC * VEC) {
                const int64_t k = k0 + (int64_t)chunk * VEC;
                const bool k_ok = k < a.J;
                for (int blk = entry_lane * group; k_ok && blk < cnt; blk += ENTRY_LANES * group) {
                    const int end = blk + group < cnt ? blk + group : cnt;
                    Vec<VEC> fiber_sum, slice_sum;
                    fiber_sum.zero();
                    slice_sum.zero();
                    int run_begin = blk;  // first entry of the slice run that slice_sum belongs to
                    for (int q0 = blk; q0 < end; q0 += D) {
                        MtRecord r[D];
                        Vec<VEC> x2[D], x1[D];
                        int close[D];  // what ends with entry q0 + u: kMtFirstFiber a fiber's share, kMtFirstSlice a slice's
#pragma unroll
                        for (int u = 0; u < D; ++u) {
                            const int q = q0 + u;
                            r[u] = s_rec[q < end ? q : blk];
                            close[u] = q + 1 >= end ? (kMtFirstFiber | kMtFirstSlice) : s_flag[q + 1];
                            if (q >= end) close[u] = 0;
                        }
#pragma unroll
                        for (int u = 0; u < D; ++u) {
                            x2[u].zero();
                            x1[u].zero();
                            if (q0 + u < end) x2[u] = load_vec<VEC>(a.X2 + (int64_t)r[u].l * a.J + k);
                            if (close[u] & kMtFirstFiber) x1[u] = load_vec<VEC>(a.X1 + (int64_t)r[u].k * a.J + k);
                        }
#pragma unroll
                        for (int u = 0; u < D; ++u) {
                            if (q0 + u >= end) continue;
                            fiber_sum.fma(r[u].val, x2[u]);
                            if (!(close[u] & kMtFirstFiber)) continue;
#pragma unroll
                            for (int v = 0; v < VEC; ++v)
                                slice_sum.v[v] = __builtin_fmaf(x1[u].v[v], fiber_sum.v[v], slice_sum.v[v]);
                            fiber_sum.zero();
                            if (!(close[u] & kMtFirstSlice)) continue;
                            if constexpr (MERGE) {
                                // a slice that starts and ends inside this lane's block has no other writer
                                const bool from_start = (s_flag[run_begin] & kMtFirstSlice) != 0;
                                if (from_start && q0 + u + 1 < end)
                                    write_out<LC, VEC>(out, r[u].i, k, true, slice_sum);
                                else
                                    merge_add<VEC, (LC >= 8)>(mb, s_slot[q0 + u], chunk * VEC, slice_sum,
                                                              chunk == 0 && (from_start || run_begin == 0), r[u].i, true);
                            } else {
                                write_out<LC, VEC>(out, r[u].i, k, false, slice_sum);  // the entry's LC chunk lanes together
                            }
                            slice_sum.zero();
                            run_begin = q0 + u + 1;
                        }
                    }
                }
                if constexpr (MERGE) {
                    __syncthreads();  // all sums of this pass are in LDS
                    merge_write_out<LC, VEC>(out, mb, k, k_ok);
                    __syncthreads();  // slots are clear again
                }
            }
        }
    }
}

namespace {

struct LaunchMttkrpNnz {
    const MttkrpArgs& a;
    int group, compute_units;
    int64_t nnz_hint;
    hipStream_t s;
    template <int G, int LC, int VEC, bool PAR, bool MERGE>
    void launch(int smem, int log2_group) const
    {
        int per_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, mttkrp_nnz_kernel<G, LC, VEC, PAR, MERGE>, kBlock,
                                                         smem) != hipSuccess || per_cu < 1)
            per_cu = 1;
        int64_t grid = (int64_t)per_cu * compute_units;
        if (nnz_hint >= 0) {
            const int64_t tiles = (nnz_hint + kMtTile - 1) / kMtTile;
            if (tiles < grid) grid = tiles > 0 ? tiles : 1;
        }
        hipLaunchKernelGGL((mttkrp_nnz_kernel<G, LC, VEC, PAR, MERGE>), dim3((unsigned)grid), dim3(kBlock), smem, s, a,
                           group, log2_group);
    }
    template <int G, int LC, int VEC, bool PAR>
    void go() const
    {
        int log2_group = 0;
        while ((1 << log2_group) < group) ++log2_group;
        // tile mode of the merge rule whenever the slots fit: the usual budget, or for small groups (whose
        // alternative is an atomic row per one or two entries) what the kernel's own 27 KB leave of the LDS
        const int smem = ((kMtTile >> log2_group) + 1) * (LC * VEC * 4 + 8);
        constexpr int kMost = 128 * 1024;
        if (smem <= kMost) {
            if (smem > 48 * 1024) {
                static const hipError_t asked = hipFuncSetAttribute(
                    reinterpret_cast<const void*>(mttkrp_nnz_kernel<G, LC, VEC, PAR, true>),
                    hipFuncAttributeMaxDynamicSharedMemorySize, kMost);
                (void)asked;
            }
            launch<G, LC, VEC, PAR, true>(smem, log2_group);
        } else {
            launch<G, LC, VEC, PAR, false>(0, log2_group);
        }
    }
};

struct LaunchMttkrpNnzPar : LaunchMttkrpNnz {
    template <int G, int LC, int VEC>
    void operator()() const { go<G, LC, VEC, true>(); }
};
struct LaunchMttkrpNnzSer : LaunchMttkrpNnz {
    template <int G, int LC, int VEC>
    void operator()() const { go<G, LC, VEC, false>(); }
};

}  // namespace

hipError_t launch_mttkrp_nnz(const MttkrpArgs& a, int g, bool parallel, int lc, int vec, int compute_units,
                             int64_t nnz_hint, hipStream_t s)
{
    bool ok;
    if (parallel) ok = dispatch_group(g, lc, vec, LaunchMttkrpNnzPar{{a, g, compute_units, nnz_hint, s}});
    else ok = dispatch_group(1, lc, vec, LaunchMttkrpNnzSer{{a, g, compute_units, nnz_hint, s}});
    if (!ok) return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace sgap
