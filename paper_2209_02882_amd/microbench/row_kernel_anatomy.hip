// What of the row-split kernel's structure costs how much?  The gather loop of
// gather_bandwidth.hip (rows of 512 bytes, two per wavefront instruction, all
// hits in L1/L2) is dressed step by step in what the SpMM kernel does around
// its gathers on a matrix of 27 entries per row, 8 rows per workgroup:
//   step 0  a resident grid, 8 loads in flight, row numbers from a generator
//   step 1  6 loads in flight, the last batch of a row 3 (27 = 4*6 + 3)
//   step 2  row numbers and values read from LDS (staged once per workgroup)
//   step 3  multiply-add with the value instead of an add
//   step 4  one short-lived workgroup per 8 rows: (column, value) pairs staged
//           from memory behind a dependent load of the row pointers, barrier,
//           27 gathers per row, exit
//   step 5  the row's 512 bytes stored at the end
//   step 6  the same tiles of 8 rows taken by a resident grid that loops over them
//   step 7  ... and requests the next tile's pairs before it multiplies the current one out
//   step 8  step 3 plus the store of step 5 (no staging from memory, no workgroup turnover)
//   step 9  step 7 with a fifth wavefront per workgroup that brings the pairs in and does nothing else
//   step 10 step 8 plus a barrier per tile; step 11 step 8 plus a tile's pairs read from memory per tile
// Standalone: hipcc --offload-arch=gfx950 -O3 row_kernel_anatomy.hip
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#include <vector>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("err %s line %d\n",hipGetErrorString(e),__LINE__); return 1;}}while(0)

constexpr int kLen = 27;     // entries per row
constexpr int kRows = 8;     // rows per workgroup of 256 lanes (32 lanes per row, 16 bytes per lane)

struct Pair { int32_t col; float val; };

// 16 bytes of a row of C: non-temporal as in the library's kernels, or (-DPLAIN_STORES) an ordinary store
__device__ __forceinline__ void store_f4(float4* p, const float4& v)
{
#ifdef PLAIN_STORES
    *p = v;
#else
    typedef float f4 __attribute__((ext_vector_type(4)));
    f4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<f4*>(p));
#endif
}

template <int D>
__device__ __forceinline__ void batch(float4& acc, const float4* __restrict__ buf, const Pair* p, int n, uint32_t chunk, bool fma,
                                      uint32_t turn = 0, uint32_t mask = 0xffffffffu)
{
    float4 v[D];
    Pair e[D];
#pragma unroll
    for (int u = 0; u < D; ++u) e[u] = u < n ? p[u] : Pair{0, 0.0f};
#pragma unroll
    for (int u = 0; u < D; ++u) v[u] = u < n ? buf[(size_t)(((uint32_t)e[u].col + turn) & mask) * 32 + chunk] : make_float4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < D; ++u) {
        const float w = fma ? e[u].val : 1.0f;
        acc.x += w * v[u].x; acc.y += w * v[u].y; acc.z += w * v[u].z; acc.w += w * v[u].w;
    }
}

// steps 0..3: resident grid, every workgroup loops `iters` times over a tile of 8 rows x 27 pairs held in LDS
template <int STEP>
__global__ __launch_bounds__(256) void resident(const float4* __restrict__ buf, float* out, uint32_t rows, int iters, uint32_t seed,
                                                float4* __restrict__ C = nullptr, const int32_t* __restrict__ cols = nullptr,
                                                const float* __restrict__ vals = nullptr)
{
    float sink = 0.0f;
    __shared__ Pair s_p[kRows * kLen];
    const uint32_t lane = threadIdx.x & 63, chunk = lane % 32, slot = threadIdx.x / 32;
    uint32_t s = (blockIdx.x * 256 + threadIdx.x / 32) * 2654435761u + seed;
    for (int i = threadIdx.x; i < kRows * kLen; i += 256) {
        uint32_t t = (blockIdx.x * 977 + i) * 2654435761u + seed;
        s_p[i] = Pair{(int32_t)(((uint64_t)(t >> 4) * rows) >> 28), 1.0f};
    }
    __syncthreads();
    float4 acc = make_float4(0, 0, 0, 0);
    for (int it = 0; it < iters; ++it) {
        if (STEP == 0) {
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                s = s * 1664525u + 1013904223u;
                v[u] = buf[(size_t)(uint32_t)(((uint64_t)(s >> 4) * rows) >> 28) * 32 + chunk];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
        } else if (STEP == 1) {
            for (int j = 0; j < kLen; j += 6) {
                float4 v[6];
                const int n = kLen - j < 6 ? kLen - j : 6;
#pragma unroll
                for (int u = 0; u < 6; ++u) {
                    s = s * 1664525u + 1013904223u;
                    v[u] = u < n ? buf[(size_t)(uint32_t)(((uint64_t)(s >> 4) * rows) >> 28) * 32 + chunk] : make_float4(0, 0, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < 6; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
            }
        } else {
            const Pair* p = s_p + slot * kLen;
            int j = 0;
            // (the row moves on by one per turn, or the loads would be taken out of the loop; rows is a power of two)
            for (; j + 6 <= kLen; j += 6) batch<6>(acc, buf, p + j, 6, chunk, STEP >= 3, (uint32_t)it, rows - 1);
            batch<3>(acc, buf, p + j, kLen - j, chunk, STEP >= 3, (uint32_t)it, rows - 1);
            if (STEP == 10) __syncthreads();  // step 8 with the waves of a workgroup meeting once per turn
            if (STEP == 11 && threadIdx.x < kRows * kLen) {
                // step 8 with a tile's pairs read from memory every turn (kept in a register, no LDS, no barrier)
                const size_t q = ((size_t)blockIdx.x + (size_t)it * gridDim.x) * (kRows * kLen) + threadIdx.x;
                sink += (float)__builtin_nontemporal_load(cols + q) + __builtin_nontemporal_load(vals + q);
            }
            if (STEP >= 8) {  // a row of C per row multiplied out, every turn another one
                store_f4(&C[((size_t)(blockIdx.x * kRows + slot) + (size_t)it * gridDim.x * kRows) * 32 + chunk], acc);
                acc = make_float4(0, 0, 0, 0);
            }
        }
    }
    if (acc.x + acc.y + acc.z + acc.w + sink == 123.456f) out[0] = acc.x;
}

// steps 4, 5: one workgroup per 8 rows
template <int STEP>
__global__ __launch_bounds__(256) void short_lived(const float4* __restrict__ buf, const int32_t* __restrict__ rowptr,
                                                   const int32_t* __restrict__ cols, const float* __restrict__ vals,
                                                   float4* __restrict__ C, float* out)
{
    __shared__ Pair s_p[kRows * kLen + 8];
    __shared__ int32_t s_rp[kRows + 1];
    const uint32_t lane = threadIdx.x & 63, chunk = lane % 32, slot = threadIdx.x / 32;
    const int64_t row0 = (int64_t)blockIdx.x * kRows;
    if (threadIdx.x <= kRows) s_rp[threadIdx.x] = rowptr[row0 + threadIdx.x];
    __syncthreads();
    const int32_t first = rowptr[row0], last = rowptr[row0 + kRows];
    for (int i = threadIdx.x; i < last - first; i += 256)
        s_p[i] = Pair{__builtin_nontemporal_load(cols + first + i), __builtin_nontemporal_load(vals + first + i)};
    __syncthreads();
    float4 acc = make_float4(0, 0, 0, 0);
    const Pair* p = s_p + (s_rp[slot] - first);
    const int len = s_rp[slot + 1] - s_rp[slot];
    int j = 0;
    for (; j + 6 <= len; j += 6) batch<6>(acc, buf, p + j, 6, chunk, true);
    if (j < len) batch<3>(acc, buf, p + j, len - j, chunk, true);
    if (STEP >= 5) store_f4(&C[(row0 + slot) * 32 + chunk], acc);
    else if (acc.x + acc.y + acc.z + acc.w == 123.456f) out[0] = acc.x;
}

// steps 6, 7: the same tiles of 8 rows, but a resident grid whose workgroups loop over tiles; step 7 requests the
// next tile's pairs (and the row pointers of the tile after it) before it multiplies the current one out
template <int STEP>
__global__ __launch_bounds__(256) void tile_loop(const float4* __restrict__ buf, const int32_t* __restrict__ rowptr,
                                                 const int32_t* __restrict__ cols, const float* __restrict__ vals,
                                                 float4* __restrict__ C, int tiles)
{
    __shared__ Pair s_p[2][kRows * kLen + 8];
    __shared__ int32_t s_rp[3][kRows + 1];
    const uint32_t lane = threadIdx.x & 63, chunk = lane % 32, slot = threadIdx.x / 32;
    const int tid = threadIdx.x;
    auto store_row = [&](int64_t row, const float4& acc) {
        store_f4(&C[row * 32 + chunk], acc);
    };
    auto multiply = [&](const Pair* sp, const int32_t* rp, int64_t row0) {
        float4 acc = make_float4(0, 0, 0, 0);
        const Pair* p = sp + (rp[slot] - rp[0]);
        const int len = rp[slot + 1] - rp[slot];
        int j = 0;
        for (; j + 6 <= len; j += 6) batch<6>(acc, buf, p + j, 6, chunk, true);
        if (j < len) batch<3>(acc, buf, p + j, len - j, chunk, true);
        store_row(row0 + slot, acc);
    };
    if (STEP == 6) {
        for (int t = blockIdx.x; t < tiles; t += gridDim.x) {
            const int64_t row0 = (int64_t)t * kRows;
            __syncthreads();
            if (tid <= kRows) s_rp[0][tid] = rowptr[row0 + tid];
            __syncthreads();
            const int32_t first = s_rp[0][0], last = s_rp[0][kRows];
            for (int i = tid; i < last - first; i += 256)
                s_p[0][i] = Pair{__builtin_nontemporal_load(cols + first + i), __builtin_nontemporal_load(vals + first + i)};
            __syncthreads();
            multiply(s_p[0], s_rp[0], row0);
        }
    } else {
        // tile j of this workgroup: t0 + j * stride.  Row pointers run two tiles ahead, pairs one.
        const int t0 = blockIdx.x, stride = gridDim.x;
        const int mine = t0 < tiles ? (tiles - t0 + stride - 1) / stride : 0;
        if (mine == 0) return;
        auto rp_load = [&](int j) { return (tid <= kRows && j < mine) ? rowptr[((int64_t)t0 + (int64_t)j * stride) * kRows + tid] : 0; };
        if (tid <= kRows) s_rp[0][tid] = rp_load(0);
        if (tid <= kRows) s_rp[1][tid] = rp_load(1);
        __syncthreads();
        Pair nx = Pair{0, 0.0f};
        {
            const int32_t first = s_rp[0][0], last = s_rp[0][kRows];
            if (tid < last - first) nx = Pair{__builtin_nontemporal_load(cols + first + tid), __builtin_nontemporal_load(vals + first + tid)};
        }
        for (int j = 0; j < mine; ++j) {
            const int b = j & 1;
            if (tid < kRows * kLen) s_p[b][tid] = nx;  // (a tile has at most 216 pairs: one per thread)
            const int32_t rp2 = rp_load(j + 2);
            __syncthreads();  // pairs of tile j and row pointers of tile j + 1 are in LDS; tile j - 1 is consumed
            if (j + 1 < mine) {
                const int32_t* rp = s_rp[(j + 1) % 3];
                const int32_t first = rp[0], last = rp[kRows];
                nx = Pair{0, 0.0f};
                if (tid < last - first) nx = Pair{__builtin_nontemporal_load(cols + first + tid), __builtin_nontemporal_load(vals + first + tid)};
            }
            multiply(s_p[b], s_rp[j % 3], ((int64_t)t0 + (int64_t)j * stride) * kRows);
            if (tid <= kRows) s_rp[(j + 2) % 3][tid] = rp2;
        }
    }
}

// step 9: as step 7, but the pairs are brought in by a fifth wavefront that does nothing else.  A wavefront's
// memory operations complete in the order they were issued, so a wavefront that has requested the next tile's
// pairs from memory cannot see its own gathers come back before them: in step 7 the request ahead hides nothing.
// Here the producer wavefront keeps the pairs of kAhead tiles in flight in its registers and writes a tile into
// LDS one turn before the four consumer wavefronts multiply it out; all five meet at one barrier per tile.
constexpr int kAhead = 4;
__global__ __launch_bounds__(320) void tile_loop_producer(const float4* __restrict__ buf, const int32_t* __restrict__ rowptr,
                                                          const int32_t* __restrict__ cols, const float* __restrict__ vals,
                                                          float4* __restrict__ C, int tiles)
{
    constexpr int kCap = kRows * kLen + 40;  // 256 pairs: four per producer lane
    __shared__ Pair s_p[2][kCap];
    __shared__ int32_t s_rp[2][kRows + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = blockIdx.x, stride = gridDim.x;
    const int mine = t0 < tiles ? (tiles - t0 + stride - 1) / stride : 0;
    auto row_of = [&](int j) { return ((int64_t)t0 + (int64_t)j * stride) * kRows; };
    if (wave == 4) {
        // tile j's row pointers are requested 2*kAhead turns ahead, its pairs kAhead turns ahead
        int32_t rp[2 * kAhead];        // lane l <= kRows holds rowptr[row0 + l] of the tiles j .. j + 2*kAhead - 1
        Pair held[kAhead][4];          // pairs of the tiles j .. j + kAhead - 1, four per lane
#pragma unroll
        for (int a = 0; a < 2 * kAhead; ++a) rp[a] = (lane <= kRows && a < mine) ? rowptr[row_of(a) + lane] : 0;
        auto request = [&](Pair (&h)[4], int32_t rpl) {
            const int32_t first = __shfl(rpl, 0, 64), last = __shfl(rpl, kRows, 64);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = lane + 64 * u;
                const int32_t q = first + (i < last - first ? i : 0);  // (a lane past the end repeats the first pair)
                h[u] = Pair{__builtin_nontemporal_load(cols + q), __builtin_nontemporal_load(vals + q)};
            }
        };
#pragma unroll
        for (int a = 0; a < kAhead; ++a)
            if (a < mine) request(held[a], rp[a]);
        for (int j0 = 0; j0 < mine + 1; j0 += 2 * kAhead) {
#pragma unroll
            for (int a = 0; a < 2 * kAhead; ++a) {  // (unrolled so that what is held stays in registers)
                const int j = j0 + a;  // writes tile j, which the consumers multiply out after the next barrier
                if (j < mine) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) s_p[j & 1][lane + 64 * u] = held[a % kAhead][u];
                    if (lane <= kRows) s_rp[j & 1][lane] = rp[a];
                }
                // what takes the freed registers: row pointers 2*kAhead tiles on, pairs kAhead tiles on
                const int32_t rp_pairs = rp[(a + kAhead) % (2 * kAhead)];
                rp[a] = (lane <= kRows && j + 2 * kAhead < mine) ? rowptr[row_of(j + 2 * kAhead) + lane] : 0;
                if (j + kAhead < mine) request(held[a % kAhead], rp_pairs);
                if (j <= mine) __syncthreads();
            }
        }
    } else {
        const uint32_t chunk = lane % 32, slot = tid / 32;
        for (int j = 0; j <= mine; ++j) {
            if (j > 0) {
                const int b = (j - 1) & 1;
                const int32_t* rpl = s_rp[b];
                float4 acc = make_float4(0, 0, 0, 0);
                const Pair* p = s_p[b] + (rpl[slot] - rpl[0]);
                const int len = rpl[slot + 1] - rpl[slot];
                int k = 0;
                for (; k + 6 <= len; k += 6) batch<6>(acc, buf, p + k, 6, chunk, true);
                if (k < len) batch<3>(acc, buf, p + k, len - k, chunk, true);
                store_f4(&C[(row_of(j - 1) + slot) * 32 + chunk], acc);
            }
            __syncthreads();
        }
    }
}

int run_producer(const float4* buf, const int32_t* rowptr, const int32_t* cols, const float* vals, float4* C, int64_t M, int per_cu, const char* what)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int tiles = (int)(M / kRows), blocks = 256 * per_cu;
    tile_loop_producer<<<blocks, 320>>>(buf, rowptr, cols, vals, C, tiles); CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int rep = 0; rep < 5; ++rep) {
        CK(hipEventRecord(e0));
        tile_loop_producer<<<blocks, 320>>>(buf, rowptr, cols, vals, C, tiles);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    const double bytes = (double)M * kLen * 512;
    printf("step 9  resident grid (%d per CU), a producer wavefront brings the pairs in, %s: %.3f ms  %7.1f GB/s  %5.1f B/clk/CU\n", per_cu,
           what, best, bytes / best / 1e6, bytes / (best * 1e-3) / 2.4e9 / 256);
    return 0;
}

// steps 12, 13: step 8 with a fifth wavefront per workgroup that only reads the pairs of the tiles from memory
// (4 bytes per lane and load, or 16), with nothing passed between it and the others: what does the stream of
// pairs cost the gathers merely by sharing their compute unit?
template <int STEP>
__global__ __launch_bounds__(320) void beside_stream(const float4* __restrict__ buf, float* out, uint32_t rows, int iters, uint32_t seed,
                                                     float4* __restrict__ C, const int32_t* __restrict__ cols, const float* __restrict__ vals)
{
    __shared__ Pair s_p[kRows * kLen];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < kRows * kLen; i += 320) {
        uint32_t t = (blockIdx.x * 977 + i) * 2654435761u + seed;
        s_p[i] = Pair{(int32_t)(((uint64_t)(t >> 4) * rows) >> 28), 1.0f};
    }
    __syncthreads();
    if (wave == 4) {
        float sink = 0.0f;
        for (int it = 0; it < iters; ++it) {
            const size_t q0 = ((size_t)blockIdx.x + (size_t)it * gridDim.x) * (kRows * kLen);
            if (STEP == 12) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int i = lane + 64 * u < kRows * kLen ? lane + 64 * u : 0;
                    sink += (float)__builtin_nontemporal_load(cols + q0 + i) + __builtin_nontemporal_load(vals + q0 + i);
                }
            } else {
                typedef int i4 __attribute__((ext_vector_type(4)));
                typedef float f4 __attribute__((ext_vector_type(4)));
                const int i = lane < kRows * kLen / 4 ? lane : 0;  // 54 lanes x 16 bytes = 216 words of each array
                const i4 c = __builtin_nontemporal_load(reinterpret_cast<const i4*>(cols + q0) + i);
                const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4*>(vals + q0) + i);
                sink += (float)(c.x + c.y + c.z + c.w) + v.x + v.y + v.z + v.w;
            }
        }
        if (sink == 123.456f) out[1] = sink;
    } else {
        const uint32_t chunk = lane % 32, slot = tid / 32;
        float4 acc = make_float4(0, 0, 0, 0);
        for (int it = 0; it < iters; ++it) {
            const Pair* p = s_p + slot * kLen;
            int j = 0;
            for (; j + 6 <= kLen; j += 6) batch<6>(acc, buf, p + j, 6, chunk, true, (uint32_t)it, rows - 1);
            batch<3>(acc, buf, p + j, kLen - j, chunk, true, (uint32_t)it, rows - 1);
            store_f4(&C[((size_t)(blockIdx.x * kRows + slot) + (size_t)it * gridDim.x * kRows) * 32 + chunk], acc);
            acc = make_float4(0, 0, 0, 0);
        }
    }
}

template <int STEP>
int run_beside(const float4* buf, float* out, float4* C, const int32_t* cols, const float* vals, int per_cu)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int blocks = 256 * per_cu, iters = 1000000 / (blocks * kRows);
    beside_stream<STEP><<<blocks, 320>>>(buf, out, 64, 4, 1, C, cols, vals); CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    beside_stream<STEP><<<blocks, 320>>>(buf, out, 64, iters, 7, C, cols, vals);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    const double bytes = (double)blocks * 256 * 16 * kLen * iters;
    printf("step %d  resident, %d workgroups per CU, window 32.8 KB, row stored, a fifth wavefront reads the pairs (%d bytes per lane): %7.1f GB/s  %5.1f B/clk/CU\n",
           STEP, per_cu, STEP == 12 ? 4 : 16, bytes / ms / 1e6, bytes / (ms * 1e-3) / 2.4e9 / 256);
    return 0;
}

template <int STEP>
int run_tile_loop(const float4* buf, const int32_t* rowptr, const int32_t* cols, const float* vals, float4* C, int64_t M, int per_cu, const char* what)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int tiles = (int)(M / kRows), blocks = 256 * per_cu;
    tile_loop<STEP><<<blocks, 256>>>(buf, rowptr, cols, vals, C, tiles); CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int rep = 0; rep < 5; ++rep) {
        CK(hipEventRecord(e0));
        tile_loop<STEP><<<blocks, 256>>>(buf, rowptr, cols, vals, C, tiles);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    const double bytes = (double)M * kLen * 512;
    printf("step %d  resident grid (%d per CU) looping over tiles of 8 rows%s, %s: %.3f ms  %7.1f GB/s  %5.1f B/clk/CU\n", STEP, per_cu,
           STEP == 7 ? ", next tile requested ahead" : "", what, best, bytes / best / 1e6, bytes / (best * 1e-3) / 2.4e9 / 256);
    return 0;
}

template <int STEP>
int run_resident(const float4* buf, float* out, uint32_t rows, int per_cu, float4* C = nullptr, const int32_t* cols = nullptr,
                 const float* vals = nullptr)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    // (step 8: blocks * 8 rows of C per turn; 69 turns of 1,792 workgroups stay inside the 1,000,000 rows)
    const int blocks = 256 * per_cu, iters = STEP == 0 ? 400 : STEP >= 8 ? 1000000 / (blocks * kRows) : 120;
    resident<STEP><<<blocks, 256>>>(buf, out, rows, 4, 1, C, cols, vals); CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    resident<STEP><<<blocks, 256>>>(buf, out, rows, iters, 7, C, cols, vals);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    const double loads = STEP == 0 ? 8.0 : (double)kLen;
    const double bytes = (double)blocks * 256 * 16 * loads * iters;
    printf("step %d  resident, %d workgroups per CU, window %6.1f KB%s: %7.1f GB/s  %5.1f B/clk/CU\n", STEP, per_cu, rows * 512 / 1e3,
           STEP == 8 ? ", a 512-byte row stored per 27 gathers" : STEP == 10 ? ", row stored, a barrier per turn" :
           STEP == 11 ? ", row stored, a tile's pairs read from memory per turn" : "",
           bytes / ms / 1e6, bytes / (ms * 1e-3) / 2.4e9 / 256);
    return 0;
}

template <int STEP>
int run_short(const float4* buf, const int32_t* rowptr, const int32_t* cols, const float* vals, float4* C, float* out, int64_t M, const char* what)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int blocks = (int)(M / kRows);
    short_lived<STEP><<<blocks, 256>>>(buf, rowptr, cols, vals, C, out); CK(hipDeviceSynchronize());
    float best = 1e30f;
    for (int rep = 0; rep < 5; ++rep) {
        CK(hipEventRecord(e0));
        short_lived<STEP><<<blocks, 256>>>(buf, rowptr, cols, vals, C, out);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        if (ms < best) best = ms;
    }
    const double bytes = (double)M * kLen * 512;
    printf("step %d  one workgroup per 8 rows, %s: %.3f ms for %lld rows  %7.1f GB/s  %5.1f B/clk/CU\n", STEP, what, best, (long long)M,
           bytes / best / 1e6, bytes / (best * 1e-3) / 2.4e9 / 256);
    return 0;
}

int main()
{
    const int64_t M = 1000000;  // rows, as the 100^3 stencil
    float4 *buf, *C; float* out; int32_t *rowptr, *cols; float* vals;
    CK(hipMalloc(&buf, (size_t)M * 512)); CK(hipMemset(buf, 0, (size_t)M * 512));
    CK(hipMalloc(&C, (size_t)M * 512)); CK(hipMalloc(&out, 16));
    CK(hipMalloc(&rowptr, (M + 1) * 4)); CK(hipMalloc(&cols, M * kLen * 4)); CK(hipMalloc(&vals, M * kLen * 4));
    std::vector<int32_t> h_rp(M + 1), h_c((size_t)M * kLen);
    std::vector<float> h_v((size_t)M * kLen, 1.0f);
    for (int64_t i = 0; i <= M; ++i) h_rp[i] = (int32_t)(i * kLen);
    CK(hipMemcpy(rowptr, h_rp.data(), (M + 1) * 4, hipMemcpyHostToDevice));
    CK(hipMemcpy(vals, h_v.data(), M * kLen * 4, hipMemcpyHostToDevice));
    for (int per_cu : {7, 8}) {
        if (run_resident<0>(buf, out, 64, per_cu)) return 1;
        if (run_resident<1>(buf, out, 64, per_cu)) return 1;
        if (run_resident<2>(buf, out, 64, per_cu)) return 1;
        if (run_resident<3>(buf, out, 64, per_cu)) return 1;
    }
    if (run_resident<3>(buf, out, 4096, 7)) return 1;
    if (run_resident<8>(buf, out, 64, 7, C)) return 1;
    if (run_resident<10>(buf, out, 64, 7, C)) return 1;
    if (run_resident<11>(buf, out, 64, 7, C, cols, vals)) return 1;
    for (int per_cu : {5, 6}) {
        if (run_beside<12>(buf, out, C, cols, vals, per_cu)) return 1;
        if (run_beside<13>(buf, out, C, cols, vals, per_cu)) return 1;
    }
    // columns of the short-lived steps: (a) 64 rows of B in all (L1), (b) the row itself and its neighbours
    // (every row of B from memory once, then L1), (c) the 27-point stencil's pattern on a 100^3 grid
    for (int pat = 0; pat < 3; ++pat) {
        for (int64_t i = 0; i < M; ++i)
            for (int j = 0; j < kLen; ++j) {
                int64_t c;
                if (pat == 0) c = (i * 7 + j) % 64;
                else if (pat == 1) c = i + (j % 3) - 1;
                else c = i + (j % 3 - 1) + 100 * ((j / 3) % 3 - 1) + 10000 * (j / 9 - 1);
                h_c[(size_t)i * kLen + j] = (int32_t)(c < 0 ? 0 : c >= M ? M - 1 : c);
            }
        CK(hipMemcpy(cols, h_c.data(), M * kLen * 4, hipMemcpyHostToDevice));
        const char* what = pat == 0 ? "64 rows of B in all" : pat == 1 ? "own row and x-neighbours" : "27-point stencil";
        if (run_short<4>(buf, rowptr, cols, vals, C, out, M, what)) return 1;
        if (run_short<5>(buf, rowptr, cols, vals, C, out, M, what)) return 1;
        for (int per_cu : {4, 5, 6}) if (run_producer(buf, rowptr, cols, vals, C, M, per_cu, what)) return 1;
        for (int per_cu : {5, 7}) {
            if (run_tile_loop<6>(buf, rowptr, cols, vals, C, M, per_cu, what)) return 1;
            if (run_tile_loop<7>(buf, rowptr, cols, vals, C, M, per_cu, what)) return 1;
        }
    }
    return 0;
}
