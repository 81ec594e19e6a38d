// C ABI of the library: argument validation, choice of kernel instance,
// launches on the caller's stream.  See include/sgap.h for the contract.
#include "../../include/sgap.h"
#include "../../include/sgap_debug.h"

#include <cstdio>
#include <cstring>
#include <initializer_list>
#include <utility>
#include <vector>

#include "sgap_common.hpp"
#include "sgap_lane_ops.hpp"
#include "sgap_tile_deal.hpp"

namespace sgap {

// ---- small kernels that belong to the boundary, not to a schedule ---------

template <int G, int LC>
__global__ void debug_group_reduce_kernel(const float* __restrict__ in, float* __restrict__ out, int r)
{
    const int lane = threadIdx.x;
    const float s = r == G ? group_tree_sum<G, LC>(in[lane]) : group_partial_sum<G, LC>(in[lane], r * LC);
    const int member = (lane / LC) % G;
    out[lane] = member % r == 0 ? s : 0.0f;
}

template <int G, int LC>
__global__ void debug_group_seg_reduce_kernel(const float* __restrict__ in, const int32_t* __restrict__ span,
                                              float* __restrict__ out)
{
    const int lane = threadIdx.x;
    out[lane] = group_seg_sum<G, LC>(in[lane], span[lane]);
}

// Streaming kernels: what the memory system delivers to a kernel that only streams (the context for the
// roofline fractions, and what the hardware traffic counters are calibrated on).  Every workgroup takes one
// contiguous run of the array, eight 16-byte accesses in flight per lane, non-temporal (measured against a
// grid-stride walk and fewer accesses in flight: 7.1-7.3 TB/s read against 5.4-6.2).
constexpr int kStreamUnroll = 8;

// the run of 16-byte elements of workgroup b out of `blocks`: [first, last)
__device__ __forceinline__ void stream_run(int64_t n4, int64_t* first, int64_t* last)
{
    const int64_t per = (n4 + gridDim.x - 1) / gridDim.x;
    *first = per * blockIdx.x < n4 ? per * blockIdx.x : n4;
    *last = *first + per < n4 ? *first + per : n4;
}

__global__ __launch_bounds__(kBlock) void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                          int64_t n)
{
    const native_f4* __restrict__ s4 = reinterpret_cast<const native_f4*>(src);
    native_f4* __restrict__ d4 = reinterpret_cast<native_f4*>(dst);
    int64_t i, last;
    stream_run(n / 4, &i, &last);
    i += threadIdx.x;
    for (; i + (kStreamUnroll - 1) * kBlock < last; i += kStreamUnroll * kBlock) {
        native_f4 t[kStreamUnroll];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) t[u] = __builtin_nontemporal_load(s4 + i + u * kBlock);
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) __builtin_nontemporal_store(t[u], d4 + i + u * kBlock);
    }
    for (; i < last; i += kBlock) __builtin_nontemporal_store(__builtin_nontemporal_load(s4 + i), d4 + i);
    if (blockIdx.x == 0)
        for (int64_t j = n / 4 * 4 + threadIdx.x; j < n; j += kBlock) dst[j] = src[j];
}

// reads n floats; a lane whose sum is exactly `never` (no input makes it so in practice) writes it to sink, so
// that the loads cannot be removed
__global__ __launch_bounds__(kBlock) void read_f32_kernel(const float* __restrict__ src, int64_t n, float never,
                                                          float* __restrict__ sink)
{
    const native_f4* __restrict__ s4 = reinterpret_cast<const native_f4*>(src);
    float sum = 0.0f;
    int64_t i, last;
    stream_run(n / 4, &i, &last);
    i += threadIdx.x;
    for (; i + (kStreamUnroll - 1) * kBlock < last; i += kStreamUnroll * kBlock) {
        native_f4 t[kStreamUnroll];
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) t[u] = __builtin_nontemporal_load(s4 + i + u * kBlock);
#pragma unroll
        for (int u = 0; u < kStreamUnroll; ++u) sum += (t[u].x + t[u].y) + (t[u].z + t[u].w);
    }
    for (; i < last; i += kBlock) {
        const native_f4 t = __builtin_nontemporal_load(s4 + i);
        sum += (t.x + t.y) + (t.z + t.w);
    }
    if (sum == never) *sink = sum;
}

__global__ __launch_bounds__(kBlock) void write_f32_kernel(float* __restrict__ dst, int64_t n, float value)
{
    native_f4* __restrict__ d4 = reinterpret_cast<native_f4*>(dst);
    const native_f4 v = {value, value, value, value};
    int64_t i, last;
    stream_run(n / 4, &i, &last);
    for (i += threadIdx.x; i < last; i += kBlock) __builtin_nontemporal_store(v, d4 + i);
    if (blockIdx.x == 0)
        for (int64_t j = n / 4 * 4 + threadIdx.x; j < n; j += kBlock) dst[j] = value;
}

// ---- sgap_validate_csr ------------------------------------------------------

static __device__ __align__(256) unsigned long long g_validate_counters[4];

__global__ __launch_bounds__(kBlock) void validate_rowptr_kernel(const int32_t* __restrict__ rowptr, int64_t M,
                                                                 int64_t nnz, unsigned long long* __restrict__ counters)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    unsigned long long bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < M; i += stride)
        if (rowptr[i] > rowptr[i + 1]) ++bad;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (rowptr[0] != 0) ++bad;
        if (rowptr[M] != nnz) ++bad;
    }
    if (bad) atomicAdd(&counters[0], bad);
}

__global__ __launch_bounds__(kBlock) void validate_columns_kernel(const int32_t* __restrict__ colidx, int64_t nnz,
                                                                  int64_t K, unsigned long long* __restrict__ counters)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    unsigned long long bad = 0;
    for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p < nnz; p += stride)
        if (colidx[p] < 0 || colidx[p] >= K) ++bad;
    if (bad) atomicAdd(&counters[1], bad);
}

// only for a rowptr that validate_rowptr_kernel found sound: every range then lies inside colidx
__global__ __launch_bounds__(kBlock) void validate_rows_kernel(const int32_t* __restrict__ rowptr,
                                                               const int32_t* __restrict__ colidx, int64_t M,
                                                               unsigned long long* __restrict__ counters)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    unsigned long long unsorted = 0, empty = 0;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < M; i += stride) {
        const int32_t b = rowptr[i], e = rowptr[i + 1];
        if (b == e) ++empty;
        for (int32_t p = b + 1; p < e; ++p)
            if (colidx[p] <= colidx[p - 1]) ++unsorted;
    }
    if (unsorted) atomicAdd(&counters[2], unsorted);
    if (empty) atomicAdd(&counters[3], empty);
}

__global__ void validate_reset_kernel(unsigned long long* counters)
{
    if (threadIdx.x < 4) counters[threadIdx.x] = 0;
}

namespace {
struct LaunchDebugReduce {
    const float* in;
    float* out;
    int r;
    hipStream_t s;
    template <int G, int LC, int VEC>
    void operator()() const
    {
        hipLaunchKernelGGL((debug_group_reduce_kernel<G, LC>), dim3(1), dim3(kWave), 0, s, in, out, r);
    }
};
struct LaunchDebugSegReduce {
    const float* in;
    const int32_t* span;
    float* out;
    hipStream_t s;
    template <int G, int LC, int VEC>
    void operator()() const
    {
        hipLaunchKernelGGL((debug_group_seg_reduce_kernel<G, LC>), dim3(1), dim3(kWave), 0, s, in, span, out);
    }
};
}  // namespace

hipError_t launch_debug_group_reduce(const float* in, float* out, int g, int r, int lc, hipStream_t s)
{
    if (!dispatch_group(g, lc, 1, LaunchDebugReduce{in, out, r, s})) return hipErrorInvalidValue;
    return hipGetLastError();
}
hipError_t launch_debug_group_seg_reduce(const float* in, const int32_t* span, float* out, int g, int lc,
                                         hipStream_t s)
{
    if (!dispatch_group(g, lc, 1, LaunchDebugSegReduce{in, span, out, s})) return hipErrorInvalidValue;
    return hipGetLastError();
}
// mode 0: copy src -> dst; 1: read src only (dst is a one-float sink); 2: write dst only
hipError_t launch_stream_f32(const float* src, float* dst, int64_t n, int mode, int compute_units, hipStream_t s)
{
    const dim3 grid((unsigned)(compute_units * 16)), block(kBlock);
    if (mode == 0) hipLaunchKernelGGL(copy_f32_kernel, grid, block, 0, s, src, dst, n);
    else if (mode == 1) hipLaunchKernelGGL(read_f32_kernel, grid, block, 0, s, src, n, -1.2345678e38f, dst);
    else hipLaunchKernelGGL(write_f32_kernel, grid, block, 0, s, dst, n, 1.0f);
    return hipGetLastError();
}

}  // namespace sgap

// ---------------------------------------------------------------------------

// Working memory of sgap_spmm_csr_cfg_static: one copy per GPU, held until the process ends.
constexpr int64_t kStaticScratchBytes = 8ll << 20;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];

namespace {

int g_schedule = SGAP_SCHED_ROW_SPLIT;
thread_local char t_last_error[256] = "";

// tuning overrides; 0 = choose automatically
int g_tile_cols = 0;
int g_xcd_remap = -1;  // -1 auto (on), 0 off, 1 on
int g_rows_per_slot = 0;
int g_sddmm_row_cache = 1;  // SDDMM parallel: keep rows of X1 in registers where the shape allows
int g_nnz_tile = 0;    // nnz-balanced serial: forced tile size, 0 = automatic
int g_persistent = 0;  // row-split: one workgroup per item keeps the rows in flight on a die close together

bool g_profile = false;
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_events;

int fail(int status, const char* fmt, const char* detail = "")
{
    std::snprintf(t_last_error, sizeof(t_last_error), fmt, detail);
    return status;
}

bool is_pow2_group(int g) { return g >= 1 && g <= 64 && (g & (g - 1)) == 0; }

int ilog2(int v)
{
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

int pow2_ceil_capped(int64_t v, int cap)
{
    int r = 1;
    while (r < cap && r < v) r *= 2;
    return r;
}

constexpr int kXcds = 8;            // accelerator dies, each with its own L2
constexpr int64_t kMaxEntries = 2147483647LL - 65535;  // 32-bit positions with room for a tile past the end
constexpr int kAutoTileCols = 128;  // 512 bytes of a B row per work item
constexpr int kAutoWindowKb = 3072;   // KiB of B per column window of the long-rows path: most of a die's 4 MiB L2
constexpr int kAutoLongRows = 8192;   // capacity of the list of long rows when the caller names none
constexpr int kMaxLongRows = 1 << 20;

int compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

// The library's choice for every knob a caller may leave open, with the process-wide overrides of
// sgap_set_tuning filled in: what the entry points without a configuration argument run with.
sgap_config config_from_globals(int schedule, int strategy, int group_size, int reduce_size)
{
    sgap_config c;
    std::memset(&c, 0, sizeof(c));
    c.schedule = schedule;
    c.strategy = strategy;
    c.group_size = group_size;
    c.reduce_size = reduce_size;
    c.tile_cols = g_tile_cols;
    c.rows_per_group = g_rows_per_slot;
    c.xcd_remap = g_xcd_remap;
    c.persistent = g_persistent;
    c.nnz_tile = g_nnz_tile;
    return c;
}

int check_config(const sgap_config& c)
{
    if (!is_pow2_group(c.group_size)) return fail(SGAP_ERR_INVALID_ARG, "group_size must be 1,2,4,8,16,32 or 64");
    if (c.strategy != SGAP_REDUCE_PARALLEL && c.strategy != SGAP_REDUCE_SERIAL)
        return fail(SGAP_ERR_INVALID_ARG, "unknown strategy");
    if (c.schedule != SGAP_SCHED_ROW_SPLIT && c.schedule != SGAP_SCHED_NNZ_BALANCED)
        return fail(SGAP_ERR_INVALID_ARG, "unknown schedule");
    if (c.reduce_size != 0 && (!is_pow2_group(c.reduce_size) || c.reduce_size > c.group_size))
        return fail(SGAP_ERR_INVALID_ARG, "reduce_size must be a power of two, 1 <= reduce_size <= group_size");
    if (c.reduce_size != 0 && c.reduce_size != c.group_size &&
        (c.schedule != SGAP_SCHED_ROW_SPLIT || c.strategy != SGAP_REDUCE_PARALLEL))
        return fail(SGAP_ERR_INVALID_ARG, "reduce_size < group_size needs the row-split schedule and the parallel strategy");
    if (c.block_size != 0 && c.block_size != 128 && c.block_size != 256 && c.block_size != 512)
        return fail(SGAP_ERR_INVALID_ARG, "block_size must be 0, 128, 256 or 512");
    if (c.tile_cols < 0) return fail(SGAP_ERR_INVALID_ARG, "tile_cols must be >= 0");
    if (c.rows_per_group < 0 || c.rows_per_group > 65536)
        return fail(SGAP_ERR_INVALID_ARG, "rows_per_group out of range");
    if (c.xcd_remap < -1 || c.xcd_remap > 1) return fail(SGAP_ERR_INVALID_ARG, "xcd_remap must be -1, 0 or 1");
    if (c.nnz_tile != 0 && c.nnz_tile != 256 && c.nnz_tile != 512 && c.nnz_tile != 1024 && c.nnz_tile != 2048)
        return fail(SGAP_ERR_INVALID_ARG, "nnz_tile must be 0, 256, 512, 1024 or 2048");
    if (c.long_row_min < 0) return fail(SGAP_ERR_INVALID_ARG, "long_row_min must be >= 0");
    if (c.window_kb < 0 || c.window_kb > (1 << 20)) return fail(SGAP_ERR_INVALID_ARG, "window_kb out of range");
    if (c.max_long_rows < 0 || c.max_long_rows > kMaxLongRows)
        return fail(SGAP_ERR_INVALID_ARG, "max_long_rows must be between 0 and 1,048,576");
    if (c.wave_rows < -1 || c.wave_rows > 1) return fail(SGAP_ERR_INVALID_ARG, "wave_rows must be -1, 0 or 1");
    return SGAP_OK;
}

int widest_vec(int64_t N, const void* p, const void* q)
{
    const uintptr_t align_bits = reinterpret_cast<uintptr_t>(p) | reinterpret_cast<uintptr_t>(q);
    if (N % 4 == 0 && (align_bits & 15) == 0) return 4;
    if (N % 2 == 0 && (align_bits & 7) == 0) return 2;
    return 1;
}

// does this call take its long rows by column windows?
bool windows_apply(const sgap_config& c, int vec)
{
    const bool whole_group = c.reduce_size == 0 || c.reduce_size == c.group_size;
    return c.long_row_min > 0 && c.schedule == SGAP_SCHED_ROW_SPLIT && whole_group && vec == 4;
}

int64_t window_bytes_of(const sgap_config& c) { return (int64_t)(c.window_kb > 0 ? c.window_kb : kAutoWindowKb) * 1024; }
int64_t long_rows_of(const sgap_config& c) { return c.max_long_rows > 0 ? c.max_long_rows : kAutoLongRows; }

int spmm_impl(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx, const float* vals,
              const float* B, float* C, const sgap_config& c, int64_t nnz_hint, void* workspace,
              int64_t workspace_bytes, void* stream)
{
    using namespace sgap;
    if (M < 0 || K < 0 || N < 0) return fail(SGAP_ERR_INVALID_ARG, "negative dimension");
    if (M > 2147483646LL || N > 2147483647LL || K > 2147483647LL)
        return fail(SGAP_ERR_INVALID_ARG, "dimension exceeds int32 index range");
    if (const int st = check_config(c)) return st;
    if (nnz_hint < -1) return fail(SGAP_ERR_INVALID_ARG, "nnz_hint must be -1 or a count");
    if (nnz_hint > kMaxEntries) return fail(SGAP_ERR_INVALID_ARG, "more stored entries than 2^31 - 65536");
    if (workspace_bytes < 0) return fail(SGAP_ERR_INVALID_ARG, "workspace_bytes must be >= 0");
    const int group_size = c.group_size;
    const int reduce_size = c.reduce_size == group_size ? 0 : c.reduce_size;
    if (M == 0 || N == 0) return SGAP_OK;
    if (!rowptr || !C) return fail(SGAP_ERR_INVALID_ARG, "rowptr and C must not be null");
    if (K > 0 && !B) return fail(SGAP_ERR_INVALID_ARG, "B must not be null when K > 0");
    if (nnz_hint > 0 && (!colidx || !vals))
        return fail(SGAP_ERR_INVALID_ARG, "colidx and vals must not be null when A has entries");

    // columns per lane (coarsening c): widest vector the shape and alignment allow
    const int vec = widest_vec(N, B, C);
    const int64_t chunks = (N + vec - 1) / vec;
    const bool windows = windows_apply(c, vec) && K > 0;
    if (windows) {
        const int64_t need = spmm_panels_workspace_bytes(K, N, window_bytes_of(c), long_rows_of(c));
        if (!workspace || workspace_bytes < need)
            return fail(SGAP_ERR_INVALID_ARG, "long_row_min > 0 needs a workspace of sgap_spmm_csr_workspace_size bytes");
        if (reinterpret_cast<uintptr_t>(workspace) & 255)
            return fail(SGAP_ERR_INVALID_ARG, "the workspace must be 256-byte aligned");
    }

    SpmmArgs a;
    a.M = M; a.K = K; a.N = N;
    a.rowptr = rowptr; a.colidx = colidx; a.vals = vals; a.B = B; a.C = C;
    a.group = group_size;
    a.log2_group = ilog2(group_size);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    // while profiling is on, a pair of events brackets everything the call enqueues
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    hipError_t err = hipSuccess;
    auto mark = [&](hipEvent_t& ev) {
        if (g_profile && hipEventCreate(&ev) == hipSuccess) hipEventRecord(ev, s);
    };
    mark(ev0);

    const bool par = c.strategy == SGAP_REDUCE_PARALLEL;
    if (c.schedule == SGAP_SCHED_ROW_SPLIT) {
        const int xcds = c.xcd_remap == 0 ? 1 : kXcds;
        const int cus = compute_units();
        const int block = c.block_size > 0 ? c.block_size : kBlock;
        const int g = par ? group_size : 1;  // lanes per row
        const double avg_row = nnz_hint > 0 ? (double)nnz_hint / (double)M : 16.0;
        // Column tile: how many columns of B/C one work item covers.
        int64_t tile_cols = c.tile_cols > 0 ? c.tile_cols : kAutoTileCols;
        if (tile_cols > N) tile_cols = N;
        tile_cols = (tile_cols + vec - 1) / vec * vec;
        const int lc = pow2_ceil_capped(tile_cols / vec, 64 / g);
        int rows_per_slot = par ? c.rows_per_group : group_size;
        if (rows_per_slot <= 0) {
            // rows a group works through per item: enough stored entries per
            // workgroup to amortise staging, few enough that neighbouring rows stay in flight together
            const int slots = block / (g * lc);
            rows_per_slot = (int)(432.0 / (avg_row * slots) + 0.5);
            if (rows_per_slot < 1) rows_per_slot = 1;
            if (rows_per_slot > 1024 / slots) rows_per_slot = 1024 / slots > 0 ? 1024 / slots : 1;
        }
        // Serial strategy in the widest lane layout: one wavefront per group_size consecutive rows (at most 63),
        // all 64 lanes on column chunks of 1, 2 or 4 columns (the widest that fills most of the lanes).  On request
        // from 48 columns on; by itself only for the rows that the window path leaves, from 192 columns on:
        // what is left there is short rows (skewed: 0.63 -> 0.37 ms for that part), while on rows of a few dozen
        // entries the narrower layout, with more rows in flight per workgroup, is faster (stencil27 at N = 256:
        // 1.27 against 1.52 ms) and 8-byte loads cost as much as 16-byte ones (N = 128: 0.62 against 0.94 ms).
        const bool wave_wanted = c.wave_rows == 1 ? N >= 48 : c.wave_rows == 0 && windows && N >= 192;
        const int wave_vec = wave_wanted && !par && reduce_size == 0 ? (N > 128 ? vec : N > 64 ? (vec < 2 ? vec : 2) : 1) : 0;
        const int wave_rows_count = group_size > 63 ? 63 : group_size;
        if (reduce_size != 0) {
            // every row receives atomic adds
            err = launch_nnz_zero_rows(a, vec, -1, s);
            if (err == hipSuccess)
                err = launch_row_split_partial(a, g, reduce_size, lc, vec, rows_per_slot, (int)tile_cols, xcds, cus,
                                               c.persistent != 0, block, s);
        } else if (windows) {
            err = launch_row_split_panels(a, g, lc, vec, wave_vec > 0 ? wave_rows_count : rows_per_slot, par,
                                          (int)tile_cols, xcds, cus, c.persistent != 0, block, wave_vec, c.long_row_min,
                                          window_bytes_of(c), workspace, long_rows_of(c), s);
        } else if (wave_vec > 0) {
            err = launch_wave_rows(a, wave_vec, wave_rows_count, xcds, nullptr, s);
        } else {
            // the parallel strategy interleaves its groups' rows; the serial strategy's lanes
            // own consecutive rows by definition
            err = launch_row_split(a, g, lc, vec, rows_per_slot, par, (int)tile_cols, xcds, cus, c.persistent != 0,
                                   block, s);
        }
    } else {
        const int lc = pow2_ceil_capped(chunks, par ? 64 / group_size : 64);
        const NnzPlan plan = par ? plan_nnz_parallel(group_size, lc, vec)
                                 : plan_nnz_serial(group_size, lc, vec, nnz_hint, compute_units(), c.nnz_tile);
        err = launch_nnz_zero_rows(a, vec, plan.merge_log2, s);
        if (err == hipSuccess)
            err = par ? launch_nnz_parallel(a, lc, vec, compute_units(), nnz_hint, s)
                      : launch_nnz_serial(a, lc, vec, plan, compute_units(), nnz_hint, s);
    }
    if (ev0) {
        mark(ev1);
        if (ev1) g_events.emplace_back(ev0, ev1); else hipEventDestroy(ev0);
    }
    if (err != hipSuccess) return fail(SGAP_ERR_HIP, "HIP launch failed: %s", hipGetErrorString(err));
    return SGAP_OK;
}

// The tuner behind sgap_autotune_csr and sgap_autotune_csr_cfg: times candidate configurations on the
// caller's operands with events on the caller's stream.  wide = false: the 28 (group size, strategy, schedule)
// points; wide = true: also the points with the reduction narrower than the tiling, the long rows by column
// windows (when the workspace is large enough) and, around the fastest point found, the tiling knobs of
// Section 7.2's space <groupSz, blockSz, tileSz, workerDimR>.
int tune_impl(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx, const float* vals,
              const float* B, float* C, int64_t nnz_hint, int reps, void* workspace, int64_t workspace_bytes, bool wide,
              sgap_tuned_point* table, int capacity, int* count, sgap_tuned_point* best, void* stream)
{
    if (reps < 1) return fail(SGAP_ERR_INVALID_ARG, "reps must be >= 1");
    if (M <= 0 || N <= 0) return fail(SGAP_ERR_INVALID_ARG, "nothing to time: M and N must be positive");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) hipEventDestroy(e0);
        return fail(SGAP_ERR_HIP, "could not create timing events");
    }
    int status = SGAP_OK;
    // one timed run of a configuration; < 0 on error
    auto timed = [&](const sgap_config& c) -> float {
        float ms = -1.0f;
        if (hipEventRecord(e0, s) != hipSuccess) status = fail(SGAP_ERR_HIP, "event record failed");
        if (status == SGAP_OK)
            status = spmm_impl(M, K, N, rowptr, colidx, vals, B, C, c, nnz_hint, workspace, workspace_bytes, stream);
        if (status == SGAP_OK && (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                                  hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
            status = fail(SGAP_ERR_HIP, "could not time a launch");
        return status == SGAP_OK ? ms : -1.0f;
    };
    sgap_tuned_point fastest;
    fastest.ms = -1.0f;
    int n = 0;
    // a configuration runs once, timed, as a warm-up and, unless that run was more than 4 times slower than the
    // best so far, `reps` more times; its time is the minimum
    auto rate = [&](const sgap_config& c) {
        if (status != SGAP_OK) return;
        // a window size the caller's workspace does not cover is not a candidate
        if (windows_apply(c, widest_vec(N, B, C)) && K > 0 &&
            (!workspace || workspace_bytes < sgap::spmm_panels_workspace_bytes(K, N, window_bytes_of(c), long_rows_of(c))))
            return;
        sgap_tuned_point pt;
        pt.config = c;
        pt.ms = timed(c);
        const bool hopeless = fastest.ms > 0.0f && pt.ms > 4.0f * fastest.ms;
        for (int r = 0; r < reps && !hopeless && status == SGAP_OK; ++r) {
            const float ms = timed(c);
            if (ms < pt.ms) pt.ms = ms;
        }
        if (status != SGAP_OK) return;
        if (table && n < capacity) table[n] = pt;
        ++n;
        if (fastest.ms < 0.0f || pt.ms < fastest.ms) fastest = pt;
    };
    for (int schedule : {SGAP_SCHED_ROW_SPLIT, SGAP_SCHED_NNZ_BALANCED})
        for (int strategy : {SGAP_REDUCE_PARALLEL, SGAP_REDUCE_SERIAL})
            for (int group = 1; group <= 64; group *= 2) rate(config_from_globals(schedule, strategy, group, 0));
    if (wide) {
        // {<1/g row, c col>, r} with r < g (Table 1's experiment)
        for (int group = 2; group <= 64; group *= 2)
            for (int r = 1; r < group; r *= 2)
                rate(config_from_globals(SGAP_SCHED_ROW_SPLIT, SGAP_REDUCE_PARALLEL, group, r));
        // long rows by column windows, if the caller brought working memory for the default list and window
        sgap_config probe = config_from_globals(SGAP_SCHED_ROW_SPLIT, SGAP_REDUCE_SERIAL, 1, 0);
        probe.long_row_min = 1024;
        const int vec = widest_vec(N, B, C);
        if (workspace && K > 0 && windows_apply(probe, vec) &&
            workspace_bytes >= sgap::spmm_panels_workspace_bytes(K, N, window_bytes_of(probe), long_rows_of(probe)) &&
            (reinterpret_cast<uintptr_t>(workspace) & 255) == 0) {
            for (int strategy : {SGAP_REDUCE_SERIAL, SGAP_REDUCE_PARALLEL})
                for (int group = 1; group <= 8; group *= 2)
                    for (int min_len : {512, 2048}) {
                        sgap_config c = config_from_globals(SGAP_SCHED_ROW_SPLIT, strategy, group, 0);
                        c.long_row_min = min_len;
                        rate(c);
                    }
        }
        // around the fastest point: workgroup size, column tile, rows per group (row-split); tile of entries
        // (nnz-balanced serial); one knob at a time, keeping what helps
        if (status == SGAP_OK) {
            auto try_values = [&](int sgap_config::*knob, std::initializer_list<int> values) {
                const sgap_config base = fastest.config;
                for (int v : values) {
                    if (base.*knob == v) continue;
                    sgap_config c = base;
                    c.*knob = v;
                    rate(c);
                }
            };
            if (fastest.config.schedule == SGAP_SCHED_ROW_SPLIT) {
                try_values(&sgap_config::block_size, {128, 512});
                try_values(&sgap_config::tile_cols, {32, 64, 256});
                if (fastest.config.strategy == SGAP_REDUCE_PARALLEL) try_values(&sgap_config::rows_per_group, {1, 2, 4, 8, 16});
                if (fastest.config.long_row_min > 0) try_values(&sgap_config::window_kb, {2048, 4096});
                if (fastest.config.strategy == SGAP_REDUCE_SERIAL) try_values(&sgap_config::wave_rows, {-1, 1});
            } else if (fastest.config.strategy == SGAP_REDUCE_SERIAL) {
                try_values(&sgap_config::nnz_tile, {512, 1024, 2048});
            }
        }
    }
    // leave the fastest point's result in C
    if (status == SGAP_OK) timed(fastest.config);
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    if (status != SGAP_OK) return status;
    *count = n;
    *best = fastest;
    return SGAP_OK;
}

}  // namespace

extern "C" {

int sgap_set_schedule(int schedule)
{
    if (schedule != SGAP_SCHED_ROW_SPLIT && schedule != SGAP_SCHED_NNZ_BALANCED)
        return fail(SGAP_ERR_INVALID_ARG, "unknown schedule");
    g_schedule = schedule;
    return SGAP_OK;
}

int sgap_get_schedule(void) { return g_schedule; }

int sgap_spmm_csr(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx, const float* vals,
                  const float* B, float* C, int group_size, int strategy, void* stream)
{
    return spmm_impl(M, K, N, rowptr, colidx, vals, B, C, config_from_globals(g_schedule, strategy, group_size, 0), -1,
                     nullptr, 0, stream);
}

int sgap_spmm_csr_ex(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx,
                     const float* vals, const float* B, float* C, int group_size, int strategy, int schedule,
                     int64_t nnz_hint, void* stream)
{
    return spmm_impl(M, K, N, rowptr, colidx, vals, B, C, config_from_globals(schedule, strategy, group_size, 0),
                     nnz_hint, nullptr, 0, stream);
}

int sgap_spmm_csr_gr(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx,
                     const float* vals, const float* B, float* C, int group_size, int reduce_size, int64_t nnz_hint,
                     void* stream)
{
    if (reduce_size < 1) return fail(SGAP_ERR_INVALID_ARG, "reduce_size must be a power of two, 1 <= reduce_size <= group_size");
    return spmm_impl(M, K, N, rowptr, colidx, vals, B, C,
                     config_from_globals(SGAP_SCHED_ROW_SPLIT, SGAP_REDUCE_PARALLEL, group_size, reduce_size), nnz_hint,
                     nullptr, 0, stream);
}

int sgap_config_init(sgap_config* config)
{
    if (!config) return fail(SGAP_ERR_INVALID_ARG, "config must not be null");
    std::memset(config, 0, sizeof(*config));
    config->schedule = SGAP_SCHED_ROW_SPLIT;
    config->strategy = SGAP_REDUCE_PARALLEL;
    config->group_size = 8;
    config->xcd_remap = -1;
    return SGAP_OK;
}

int64_t sgap_spmm_csr_workspace_size(int64_t M, int64_t K, int64_t N, const sgap_config* config)
{
    if (!config || M < 0 || K < 0 || N < 0) {
        fail(SGAP_ERR_INVALID_ARG, "bad arguments");
        return -1;
    }
    if (check_config(*config) != SGAP_OK) return -1;
    // (the vector width is not known without the operands: sized as if the window path applied)
    if (config->long_row_min == 0 || config->schedule != SGAP_SCHED_ROW_SPLIT || N % 4 != 0 || K == 0 || N == 0) return 0;
    if (config->reduce_size != 0 && config->reduce_size != config->group_size) return 0;
    return sgap::spmm_panels_workspace_bytes(K, N, window_bytes_of(*config), long_rows_of(*config));
}

int sgap_spmm_csr_cfg(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx,
                      const float* vals, const float* B, float* C, const sgap_config* config, int64_t nnz_hint,
                      void* workspace, int64_t workspace_bytes, void* stream)
{
    if (!config) return fail(SGAP_ERR_INVALID_ARG, "config must not be null");
    return spmm_impl(M, K, N, rowptr, colidx, vals, B, C, *config, nnz_hint, workspace, workspace_bytes, stream);
}

int sgap_spmm_csr_cfg_static(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx,
                             const float* vals, const float* B, float* C, const sgap_config* config,
                             int64_t nnz_hint, void* stream)
{
    if (!config) return fail(SGAP_ERR_INVALID_ARG, "config must not be null");
    // what the call would ask of a caller's workspace must fit the built-in array
    const int64_t need = sgap_spmm_csr_workspace_size(M, K, N, config);
    if (need < 0) return SGAP_ERR_INVALID_ARG;
    if (need > kStaticScratchBytes) {
        char detail[160];
        std::snprintf(detail, sizeof(detail),
                      "this shape and configuration need %lld bytes of working memory; the built-in array holds %lld",
                      (long long)need, (long long)kStaticScratchBytes);
        return fail(SGAP_ERR_UNSUPPORTED, "%s", detail);
    }
    // this GPU's copy of the array: looked up once per device, with that device current
    // (the array's name is a host-side stand-in, not a device address)
    constexpr int kMaxDevices = 64;
    static void* per_device[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return fail(SGAP_ERR_HIP, "could not tell the current device");
    if (!per_device[dev]) {
        void* ptr = nullptr;
        const hipError_t err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch));
        if (err != hipSuccess || !ptr)
            return fail(SGAP_ERR_HIP, "could not locate the built-in working memory: %s", hipGetErrorString(err));
        per_device[dev] = ptr;
    }
    // (nothing has to be cleared here: the first kernel of the window path resets the header of the
    // workspace, the only part it reads before writing, on every call)
    return spmm_impl(M, K, N, rowptr, colidx, vals, B, C, *config, nnz_hint, per_device[dev], kStaticScratchBytes, stream);
}

static int sddmm_impl(int64_t M, int64_t K, int64_t J, const int32_t* rowptr, const int32_t* colidx,
                      const float* vals, const float* X1, const float* X2T, float* out_vals, int group_size,
                      int strategy, int64_t nnz_hint, int long_row_min, int window_kb, int max_long_rows,
                      void* workspace, int64_t workspace_bytes, void* stream)
{
    using namespace sgap;
    if (M < 0 || K < 0 || J < 0) return fail(SGAP_ERR_INVALID_ARG, "negative dimension");
    if (M > 2147483646LL || J > 2147483647LL || K > 2147483647LL)
        return fail(SGAP_ERR_INVALID_ARG, "dimension exceeds int32 index range");
    if (!is_pow2_group(group_size)) return fail(SGAP_ERR_INVALID_ARG, "group_size must be 1,2,4,8,16,32 or 64");
    if (strategy != SGAP_REDUCE_PARALLEL && strategy != SGAP_REDUCE_SERIAL)
        return fail(SGAP_ERR_INVALID_ARG, "unknown strategy");
    if (nnz_hint < -1) return fail(SGAP_ERR_INVALID_ARG, "nnz_hint must be -1 or a count");
    if (nnz_hint > kMaxEntries) return fail(SGAP_ERR_INVALID_ARG, "more stored entries than 2^31 - 65536");
    if (long_row_min < 0 || window_kb < 0 || window_kb > (1 << 20) || max_long_rows < 0 || max_long_rows > kMaxLongRows ||
        workspace_bytes < 0)
        return fail(SGAP_ERR_INVALID_ARG, "bad long-row arguments");
    if (M == 0 || nnz_hint == 0) return SGAP_OK;
    if (!rowptr) return fail(SGAP_ERR_INVALID_ARG, "rowptr must not be null");
    if (!colidx || !vals || !out_vals) {
        // arrays of no entries may be null; a matrix with entries cannot come without them
        if (nnz_hint > 0) return fail(SGAP_ERR_INVALID_ARG, "colidx, vals and out_vals must not be null when A has entries");
        return SGAP_OK;
    }
    if (J > 0 && (!X1 || !X2T)) return fail(SGAP_ERR_INVALID_ARG, "X1 and X2T must not be null when J > 0");

    const uintptr_t align_bits = reinterpret_cast<uintptr_t>(X1) | reinterpret_cast<uintptr_t>(X2T);
    int vec = 1;
    if (J % 4 == 0 && (align_bits & 15) == 0) vec = 4;
    else if (J % 2 == 0 && (align_bits & 7) == 0) vec = 2;

    SpmmArgs a;
    a.M = M; a.K = K; a.N = J;
    a.rowptr = rowptr; a.colidx = colidx; a.vals = vals; a.B = X2T; a.C = nullptr;
    a.group = group_size;
    a.log2_group = ilog2(group_size);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    auto mark = [&](hipEvent_t& ev) {
        if (g_profile && hipEventCreate(&ev) == hipSuccess) hipEventRecord(ev, s);
    };
    mark(ev0);
    const bool par = strategy == SGAP_REDUCE_PARALLEL;
    hipError_t err;
    if (long_row_min > 0 && vec == 4 && J >= 32 && J <= 256 && K > 0) {
        const int64_t window_bytes = (int64_t)(window_kb > 0 ? window_kb : 2048) * 1024;
        const int64_t cap = max_long_rows > 0 ? max_long_rows : kAutoLongRows;
        if (!workspace || workspace_bytes < sddmm_panels_workspace_bytes(K, J, window_bytes, cap) ||
            (reinterpret_cast<uintptr_t>(workspace) & 255)) {
            if (ev0) hipEventDestroy(ev0);
            return fail(SGAP_ERR_INVALID_ARG,
                        "long_row_min > 0 needs a 256-byte aligned workspace of sgap_sddmm_csr_workspace_size bytes");
        }
        err = launch_sddmm_panels(a, X1, out_vals, par ? group_size : 1, par ? 0 : group_size,
                                  g_xcd_remap == 0 ? 1 : kXcds, compute_units(), nnz_hint, long_row_min, window_bytes,
                                  workspace, cap, s);
    } else
        err = launch_sddmm(a, X1, out_vals, par ? group_size : 1, par ? 0 : group_size, vec, g_sddmm_row_cache != 0,
                           compute_units(), nnz_hint, s);
    if (ev0) {
        mark(ev1);
        if (ev1) g_events.emplace_back(ev0, ev1); else hipEventDestroy(ev0);
    }
    if (err != hipSuccess) return fail(SGAP_ERR_HIP, "HIP launch failed: %s", hipGetErrorString(err));
    return SGAP_OK;
}

int sgap_sddmm_csr(int64_t M, int64_t K, int64_t J, const int32_t* rowptr, const int32_t* colidx, const float* vals,
                   const float* X1, const float* X2T, float* out_vals, int group_size, int strategy, int64_t nnz_hint,
                   void* stream)
{
    return sddmm_impl(M, K, J, rowptr, colidx, vals, X1, X2T, out_vals, group_size, strategy, nnz_hint, 0, 0, 0, nullptr,
                      0, stream);
}

int sgap_sddmm_csr_windows(int64_t M, int64_t K, int64_t J, const int32_t* rowptr, const int32_t* colidx,
                           const float* vals, const float* X1, const float* X2T, float* out_vals, int group_size,
                           int strategy, int64_t nnz_hint, int long_row_min, int window_kb, int max_long_rows,
                           void* workspace, int64_t workspace_bytes, void* stream)
{
    return sddmm_impl(M, K, J, rowptr, colidx, vals, X1, X2T, out_vals, group_size, strategy, nnz_hint, long_row_min,
                      window_kb, max_long_rows, workspace, workspace_bytes, stream);
}

int64_t sgap_sddmm_csr_workspace_size(int64_t K, int64_t J, int window_kb, int max_long_rows)
{
    if (K < 0 || J < 0 || window_kb < 0 || window_kb > (1 << 20) || max_long_rows < 0 || max_long_rows > kMaxLongRows) {
        fail(SGAP_ERR_INVALID_ARG, "bad arguments");
        return -1;
    }
    if (K == 0 || J % 4 != 0 || J < 32 || J > 256) return 0;  // the window path does not apply
    return sgap::sddmm_panels_workspace_bytes(K, J, (int64_t)(window_kb > 0 ? window_kb : 2048) * 1024,
                                              max_long_rows > 0 ? max_long_rows : kAutoLongRows);
}

int sgap_ttm_csf(int64_t F, int64_t K, int64_t L, const int32_t* eptr, const int32_t* eidx, const float* vals,
                 const float* X1, float* Yf, int group_size, int strategy, int schedule, int64_t nnz_hint,
                 void* stream)
{
    // the reduction over the entries of a fiber is the SpMM reduction over the entries of a row
    return spmm_impl(F, K, L, eptr, eidx, vals, X1, Yf, config_from_globals(schedule, strategy, group_size, 0), nnz_hint,
                     nullptr, 0, stream);
}

int sgap_mttkrp_csf(int64_t I, int64_t K, int64_t L, int64_t J, const int32_t* fptr, const int32_t* fidx,
                    const int32_t* eptr, const int32_t* eidx, const float* vals, const float* X1, const float* X2,
                    float* Y, int group_size, int strategy, void* stream)
{
    return sgap_mttkrp_csf_ex(I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2, Y, group_size, strategy,
                              SGAP_SCHED_ROW_SPLIT, -1, stream);
}

int sgap_mttkrp_csf_ex(int64_t I, int64_t K, int64_t L, int64_t J, const int32_t* fptr, const int32_t* fidx,
                       const int32_t* eptr, const int32_t* eidx, const float* vals, const float* X1, const float* X2,
                       float* Y, int group_size, int strategy, int schedule, int64_t nnz_hint, void* stream)
{
    using namespace sgap;
    if (schedule != SGAP_SCHED_ROW_SPLIT && schedule != SGAP_SCHED_NNZ_BALANCED)
        return fail(SGAP_ERR_INVALID_ARG, "unknown schedule");
    if (I < 0 || K < 0 || L < 0 || J < 0) return fail(SGAP_ERR_INVALID_ARG, "negative dimension");
    if (I > 2147483646LL || K > 2147483647LL || L > 2147483647LL || J > 2147483647LL)
        return fail(SGAP_ERR_INVALID_ARG, "dimension exceeds int32 index range");
    if (!is_pow2_group(group_size)) return fail(SGAP_ERR_INVALID_ARG, "group_size must be 1,2,4,8,16,32 or 64");
    if (strategy != SGAP_REDUCE_PARALLEL && strategy != SGAP_REDUCE_SERIAL)
        return fail(SGAP_ERR_INVALID_ARG, "unknown strategy");
    if (I == 0 || J == 0) return SGAP_OK;
    if (!fptr || !Y) return fail(SGAP_ERR_INVALID_ARG, "fptr and Y must not be null");
    if (K > 0 && L > 0 && (!X1 || !X2)) return fail(SGAP_ERR_INVALID_ARG, "X1 and X2 must not be null");
    // (fidx, eptr, eidx and vals are read only for fibers that fptr announces)

    const uintptr_t align_bits =
        reinterpret_cast<uintptr_t>(X1) | reinterpret_cast<uintptr_t>(X2) | reinterpret_cast<uintptr_t>(Y);
    int vec = 1;
    if (J % 4 == 0 && (align_bits & 15) == 0) vec = 4;
    else if (J % 2 == 0 && (align_bits & 7) == 0) vec = 2;
    const bool par = strategy == SGAP_REDUCE_PARALLEL;
    const int g = par ? group_size : 1;
    const int lc = pow2_ceil_capped((J + vec - 1) / vec, 64 / g);
    // parallel: about 16 slices per workgroup, enough to pay for bringing a block's slice pointers,
    // fibers and entries into LDS (more lose occupancy to the LDS copies); serial: group_size slices per lane
    const int slots = 256 / (g * lc);
    const int rows_per_slot = !par ? group_size : g_rows_per_slot > 0 ? g_rows_per_slot : (slots >= 16 ? 1 : 16 / slots);
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    auto mark = [&](hipEvent_t& ev) {
        if (g_profile && hipEventCreate(&ev) == hipSuccess) hipEventRecord(ev, s);
    };
    mark(ev0);
    hipError_t err;
    if (schedule == SGAP_SCHED_NNZ_BALANCED) {
        // every run's sum is added into Y: all of Y starts at zero (zero_rows_kernel with "every row")
        SpmmArgs z{};
        z.M = I; z.K = K; z.N = J; z.rowptr = fptr; z.C = Y;
        err = launch_nnz_zero_rows(z, vec, -1, s);
        if (err == hipSuccess) {
            const MttkrpArgs m{I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2, Y};
            const int lanes = pow2_ceil_capped((J + vec - 1) / vec, par ? 64 / group_size : 64);
            err = launch_mttkrp_nnz(m, group_size, par, lanes, vec, compute_units(), nnz_hint, s);
        }
    } else
        err = launch_mttkrp(I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2, Y, g, rows_per_slot, par, lc, vec,
                            g_xcd_remap == 0 ? 1 : kXcds, s);
    if (ev0) {
        mark(ev1);
        if (ev1) g_events.emplace_back(ev0, ev1); else hipEventDestroy(ev0);
    }
    if (err != hipSuccess) return fail(SGAP_ERR_HIP, "HIP launch failed: %s", hipGetErrorString(err));
    return SGAP_OK;
}

int sgap_autotune_csr(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx,
                      const float* vals, const float* B, float* C, int64_t nnz_hint, int reps, sgap_point_time* table,
                      sgap_point_time* best, void* stream)
{
    if (!best) return fail(SGAP_ERR_INVALID_ARG, "best must not be null");
    std::vector<sgap_tuned_point> points(SGAP_NUM_POINTS);
    sgap_tuned_point fastest;
    int count = 0;
    const int status = tune_impl(M, K, N, rowptr, colidx, vals, B, C, nnz_hint, reps, nullptr, 0, false, points.data(),
                                 SGAP_NUM_POINTS, &count, &fastest, stream);
    if (status != SGAP_OK) return status;
    for (int i = 0; i < count && table; ++i)
        table[i] = {points[i].config.group_size, points[i].config.strategy, points[i].config.schedule, points[i].ms};
    *best = {fastest.config.group_size, fastest.config.strategy, fastest.config.schedule, fastest.ms};
    return SGAP_OK;
}

int sgap_autotune_csr_cfg(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colidx,
                          const float* vals, const float* B, float* C, int64_t nnz_hint, int reps, void* workspace,
                          int64_t workspace_bytes, sgap_tuned_point* table, int capacity, int* count,
                          sgap_tuned_point* best, void* stream)
{
    if (!best) return fail(SGAP_ERR_INVALID_ARG, "best must not be null");
    if (capacity < 0 || (capacity > 0 && !table)) return fail(SGAP_ERR_INVALID_ARG, "bad table arguments");
    if (workspace_bytes < 0) return fail(SGAP_ERR_INVALID_ARG, "workspace_bytes must be >= 0");
    int n = 0;
    const int status = tune_impl(M, K, N, rowptr, colidx, vals, B, C, nnz_hint, reps, workspace, workspace_bytes, true,
                                 table, capacity, &n, best, stream);
    if (count) *count = n;
    return status;
}

const char* sgap_status_string(int status)
{
    switch (status) {
        case SGAP_OK: return "ok";
        case SGAP_ERR_INVALID_ARG: return "invalid argument";
        case SGAP_ERR_UNSUPPORTED: return "unsupported";
        case SGAP_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char* sgap_last_error(void) { return t_last_error; }

int sgap_version(void) { return 100; }

int sgap_set_tuning(int knob, int value)
{
    switch (knob) {
        case SGAP_TUNE_TILE_COLS:
            if (value < 0) return fail(SGAP_ERR_INVALID_ARG, "tile_cols must be >= 0");
            g_tile_cols = value;
            return SGAP_OK;
        case SGAP_TUNE_XCD_REMAP:
            if (value < -1 || value > 1) return fail(SGAP_ERR_INVALID_ARG, "xcd_remap must be -1, 0 or 1");
            g_xcd_remap = value;
            return SGAP_OK;
        case SGAP_TUNE_PERSISTENT:
            g_persistent = value != 0;
            return SGAP_OK;
        case SGAP_TUNE_SDDMM_ROW_CACHE:
            g_sddmm_row_cache = value != 0;
            return SGAP_OK;
        case SGAP_TUNE_NNZ_TILE:
            if (value != 0 && value != 256 && value != 512 && value != 1024 && value != 2048)
                return fail(SGAP_ERR_INVALID_ARG, "nnz tile must be 0, 256, 512, 1024 or 2048");
            g_nnz_tile = value;
            return SGAP_OK;
        case SGAP_TUNE_ROWS_PER_GROUP:
            if (value < 0 || value > 65536) return fail(SGAP_ERR_INVALID_ARG, "rows per group out of range");
            g_rows_per_slot = value;
            return SGAP_OK;
        default:
            return fail(SGAP_ERR_INVALID_ARG, "unknown tuning knob");
    }
}

int sgap_profile_enable(int on)
{
    g_profile = on != 0;
    return SGAP_OK;
}

int sgap_profile_collect(double* total_ms, int* count)
{
    double total = 0.0;
    int n = 0;
    int status = SGAP_OK;
    for (auto& ev : g_events) {
        float ms = 0.0f;
        if (hipEventSynchronize(ev.second) == hipSuccess && hipEventElapsedTime(&ms, ev.first, ev.second) == hipSuccess) {
            total += ms;
            ++n;
        } else {
            status = fail(SGAP_ERR_HIP, "could not read profiling events");
        }
        hipEventDestroy(ev.first);
        hipEventDestroy(ev.second);
    }
    g_events.clear();
    if (total_ms) *total_ms = total;
    if (count) *count = n;
    return status;
}

int sgap_debug_group_reduce(const float* in, float* out, int group_size, int lanes_per_row, void* stream)
{
    return sgap_debug_group_partial_reduce(in, out, group_size, group_size, lanes_per_row, stream);
}

int sgap_debug_group_partial_reduce(const float* in, float* out, int group_size, int reduce_size, int lanes_per_row,
                                    void* stream)
{
    if (!in || !out || !is_pow2_group(group_size) || !is_pow2_group(lanes_per_row) ||
        group_size * lanes_per_row > 64 || !is_pow2_group(reduce_size) || reduce_size > group_size)
        return fail(SGAP_ERR_INVALID_ARG, "bad group layout");
    hipError_t err = sgap::launch_debug_group_reduce(in, out, group_size, reduce_size, lanes_per_row,
                                                     reinterpret_cast<hipStream_t>(stream));
    if (err != hipSuccess) return fail(SGAP_ERR_HIP, "HIP launch failed: %s", hipGetErrorString(err));
    return SGAP_OK;
}

int sgap_debug_group_seg_reduce(const float* in, const int32_t* span, float* out, int group_size, int lanes_per_row,
                                void* stream)
{
    if (!in || !span || !out || !is_pow2_group(group_size) || !is_pow2_group(lanes_per_row) ||
        group_size * lanes_per_row > 64)
        return fail(SGAP_ERR_INVALID_ARG, "bad group layout");
    hipError_t err = sgap::launch_debug_group_seg_reduce(in, span, out, group_size, lanes_per_row,
                                                         reinterpret_cast<hipStream_t>(stream));
    if (err != hipSuccess) return fail(SGAP_ERR_HIP, "HIP launch failed: %s", hipGetErrorString(err));
    return SGAP_OK;
}

int64_t sgap_debug_tile_deal(int64_t tiles, int grid, int block, int64_t* out_tiles, int64_t capacity)
{
    if (tiles < 0 || grid < 1 || block < 0 || block >= grid || capacity < 0 || (capacity > 0 && !out_tiles)) {
        fail(SGAP_ERR_INVALID_ARG, "bad tile deal arguments");
        return -1;
    }
    const sgap::TileDeal deal(tiles, (uint32_t)block, (uint32_t)grid);
    for (int64_t j = 0; j < deal.mine && j < capacity; ++j) out_tiles[j] = deal.tile(j);
    return deal.mine;
}

int sgap_debug_plan_nnz_serial(int group_size, int lanes_per_row, int cols_per_lane, int64_t nnz_hint,
                               int compute_units_, int forced_tile, int* tile, int* merge_on_chip, int* lanes_used)
{
    if (!is_pow2_group(group_size) || !is_pow2_group(lanes_per_row) ||
        (cols_per_lane != 1 && cols_per_lane != 2 && cols_per_lane != 4) || compute_units_ < 1 || !tile ||
        !merge_on_chip)
        return fail(SGAP_ERR_INVALID_ARG, "bad plan arguments");
    const sgap::NnzPlan p =
        sgap::plan_nnz_serial(group_size, lanes_per_row, cols_per_lane, nnz_hint, compute_units_, forced_tile);
    *tile = p.tile;
    *merge_on_chip = p.merge ? 1 : 0;
    if (lanes_used) *lanes_used = p.lc;
    return SGAP_OK;
}

int64_t sgap_reorder_rows_workspace_size(int64_t M)
{
    if (M < 0) {
        fail(SGAP_ERR_INVALID_ARG, "negative size");
        return -1;
    }
    return sgap::reorder_workspace_bytes(M);
}

__global__ void first_rowptr_kernel(int32_t* rowptr_out) { rowptr_out[0] = 0; }

int sgap_reorder_rows_csr(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colidx, const float* vals,
                          int order, int32_t* perm, int32_t* rowptr_out, int32_t* colidx_out, float* vals_out,
                          void* workspace, int64_t workspace_bytes, void* stream)
{
    using namespace sgap;
    if (M < 0 || K < 0) return fail(SGAP_ERR_INVALID_ARG, "negative size");
    if (M > 2147483646LL) return fail(SGAP_ERR_INVALID_ARG, "M exceeds the int32 row range");
    if (order != SGAP_ORDER_BY_FIRST_COLUMN && order != SGAP_ORDER_BY_LENGTH)
        return fail(SGAP_ERR_INVALID_ARG, "unknown row order");
    if (!rowptr || !rowptr_out) return fail(SGAP_ERR_INVALID_ARG, "rowptr and rowptr_out must not be null");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    if (M == 0) {
        hipLaunchKernelGGL(first_rowptr_kernel, dim3(1), dim3(1), 0, s, rowptr_out);
        const hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return fail(SGAP_ERR_HIP, "HIP launch failed: %s", hipGetErrorString(e0));
        return SGAP_OK;
    }
    if (K < 1) return fail(SGAP_ERR_INVALID_ARG, "K must be positive when the matrix has rows");
    if (!perm) return fail(SGAP_ERR_INVALID_ARG, "perm must not be null");
    if (!workspace || workspace_bytes < reorder_workspace_bytes(M) || (reinterpret_cast<uintptr_t>(workspace) & 15))
        return fail(SGAP_ERR_INVALID_ARG, "workspace missing, misaligned or smaller than sgap_reorder_rows_workspace_size");
    const hipError_t err = launch_reorder_rows(M, K, rowptr, colidx, vals, order == SGAP_ORDER_BY_LENGTH, perm,
                                               rowptr_out, colidx_out, vals_out, workspace, compute_units(), s);
    if (err != hipSuccess) return fail(SGAP_ERR_HIP, "HIP launch failed: %s", hipGetErrorString(err));
    return SGAP_OK;
}

int sgap_validate_csr(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colidx, int64_t nnz, int64_t* report,
                      void* stream)
{
    using namespace sgap;
    if (M < 0 || K < 0 || nnz < 0) return fail(SGAP_ERR_INVALID_ARG, "negative size");
    if (M > 2147483646LL || nnz > 2147483647LL) return fail(SGAP_ERR_INVALID_ARG, "size exceeds int32 index range");
    if (!report) return fail(SGAP_ERR_INVALID_ARG, "report must not be null");
    if (!rowptr) return fail(SGAP_ERR_INVALID_ARG, "rowptr must not be null");
    if (nnz > 0 && !colidx) return fail(SGAP_ERR_INVALID_ARG, "colidx must not be null when nnz > 0");
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    // this GPU's copy of the counters (the symbol's name is a host-side stand-in, not a device address)
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(g_validate_counters)) != hipSuccess)
        return fail(SGAP_ERR_HIP, "could not locate the counters");
    unsigned long long* counters = static_cast<unsigned long long*>(sym);
    const unsigned grid = (unsigned)(compute_units() * 8);
    unsigned long long host[4] = {0, 0, 0, 0};
    hipLaunchKernelGGL(validate_reset_kernel, dim3(1), dim3(kWave), 0, s, counters);
    hipLaunchKernelGGL(validate_rowptr_kernel, dim3(grid), dim3(kBlock), 0, s, rowptr, M, nnz, counters);
    if (nnz > 0) hipLaunchKernelGGL(validate_columns_kernel, dim3(grid), dim3(kBlock), 0, s, colidx, nnz, K, counters);
    hipError_t err = hipGetLastError();
    if (err == hipSuccess) err = hipMemcpyAsync(host, counters, sizeof(host), hipMemcpyDeviceToHost, s);
    if (err == hipSuccess) err = hipStreamSynchronize(s);
    if (err != hipSuccess) return fail(SGAP_ERR_HIP, "HIP error: %s", hipGetErrorString(err));
    report[0] = (int64_t)host[0];
    report[1] = (int64_t)host[1];
    report[2] = report[3] = -1;
    if (host[0] == 0) {
        hipLaunchKernelGGL(validate_rows_kernel, dim3(grid), dim3(kBlock), 0, s, rowptr, colidx, M, counters);
        err = hipGetLastError();
        if (err == hipSuccess) err = hipMemcpyAsync(host, counters, sizeof(host), hipMemcpyDeviceToHost, s);
        if (err == hipSuccess) err = hipStreamSynchronize(s);
        if (err != hipSuccess) return fail(SGAP_ERR_HIP, "HIP error: %s", hipGetErrorString(err));
        report[2] = (int64_t)host[2];
        report[3] = (int64_t)host[3];
    }
    return SGAP_OK;
}

int sgap_stream_f32(const float* src, float* dst, int64_t n, int mode, void* stream)
{
    if (mode < 0 || mode > 2) return fail(SGAP_ERR_INVALID_ARG, "mode must be 0 (copy), 1 (read) or 2 (write)");
    if (n < 0 || (n > 0 && ((mode != 2 && !src) || !dst))) return fail(SGAP_ERR_INVALID_ARG, "bad stream arguments");
    if (n == 0) return SGAP_OK;
    if ((reinterpret_cast<uintptr_t>(mode != 2 ? src : nullptr) | reinterpret_cast<uintptr_t>(mode != 1 ? dst : nullptr)) & 15)
        return fail(SGAP_ERR_INVALID_ARG, "stream buffers must be 16-byte aligned");
    hipError_t err = sgap::launch_stream_f32(src, dst, n, mode, compute_units(), reinterpret_cast<hipStream_t>(stream));
    if (err != hipSuccess) return fail(SGAP_ERR_HIP, "HIP launch failed: %s", hipGetErrorString(err));
    return SGAP_OK;
}

int sgap_copy_f32(const float* src, float* dst, int64_t n, void* stream) { return sgap_stream_f32(src, dst, n, 0, stream); }

}  // extern "C"
