// Wave-uniform gathers: one wavefront works on one row of A at a time and its
// 64 lanes hold 64 neighbouring column chunks of the dense operand (LC = 64 in
// the lane layout of sgap_lane_ops.hpp, the paper's coarsening factor c = VEC
// columns per lane, Section 3.1).  Every lane then wants the same stored entry:
// 64 entries are fetched with one coalesced load (one per lane, the next 64
// requested before the current ones are worked through), and an entry's
// (column, value) pair is read out of its lane into scalar registers, so that
// the address of its row of B costs one scalar multiply, the load needs no
// vector register for an address, and the value enters the multiply-add as a
// scalar operand.  (Reading the pairs with scalar loads instead, eight at a
// time, puts a scalar-cache round trip in front of every round of gathers:
// 1.5x slower on both kernels that use this.)
#pragma once
#include "sgap_common.hpp"

namespace sgap {

typedef uint32_t raw_u2 __attribute__((ext_vector_type(2)));
typedef uint32_t raw_u4 __attribute__((ext_vector_type(4)));

// Rows of B addressed by a wave-uniform column.  OFF32 (B below 4 GB): a buffer
// load with the column's byte offset in a scalar register and the lane's chunk
// offset in one vector register that never changes; else 64-bit addresses.
template <int VEC, bool OFF32>
struct UniformRows {
    __amdgpu_buffer_rsrc_t rsrc;
    uint32_t lane_off;   // byte offset of this lane's chunk inside a row
    uint32_t row_bytes;
    const float* B;
    int64_t N, k;
    __device__ __forceinline__ UniformRows(const float* B_, int64_t K, int64_t N_, int64_t k_)
        : lane_off((uint32_t)(k_ * 4)), row_bytes((uint32_t)(N_ * 4)), B(B_), N(N_), k(k_)
    {
        // raw buffer over all of B: base, stride 0, extent in bytes, 32-bit untyped data
        if constexpr (OFF32)
            rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(B_), 0, (int)(uint32_t)(K * N_ * 4), 0x00020000);
    }
    // col is the same in all lanes
    __device__ __forceinline__ Vec<VEC> load(int32_t col) const
    {
        Vec<VEC> r;
        if constexpr (OFF32) {
            const uint32_t soff = (uint32_t)col * row_bytes;
            if constexpr (VEC == 4) {
                const raw_u4 t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, lane_off, soff, 0);
                const uint32_t x = t.x, y = t.y, z = t.z, w = t.w;  // scalars first: bit_cast of a vector element misreads
                r.v[0] = __builtin_bit_cast(float, x); r.v[1] = __builtin_bit_cast(float, y);
                r.v[2] = __builtin_bit_cast(float, z); r.v[3] = __builtin_bit_cast(float, w);
            } else if constexpr (VEC == 2) {
                const raw_u2 t = __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane_off, soff, 0);
                const uint32_t x = t.x, y = t.y;
                r.v[0] = __builtin_bit_cast(float, x); r.v[1] = __builtin_bit_cast(float, y);
            } else {
                const uint32_t x = __builtin_amdgcn_raw_buffer_load_b32(rsrc, lane_off, soff, 0);
                r.v[0] = __builtin_bit_cast(float, x);
            }
        } else {
            r = load_vec<VEC>(B + ((int64_t)col * N + k));
        }
        return r;
    }
};

// 64 stored entries, one per lane: lane j holds entry base + j (nothing beyond `end`).
struct EntryChunk {
    int32_t col;
    int32_t val;  // the bits of the fp32 value
};

// Coalesced streaming load of the entries q0 + lane < q1 (q0, q1 the same in all lanes).
__device__ __forceinline__ EntryChunk load_chunk(const int32_t* __restrict__ colidx, const float* __restrict__ vals,
                                                 int32_t q0, int32_t q1, int lane)
{
    EntryChunk ch;
    ch.col = 0;
    ch.val = 0;
    if (q0 + lane < q1) {
        ch.col = load_stream(colidx + q0 + lane);
        ch.val = __float_as_int(load_stream(vals + q0 + lane));
    }
    return ch;
}

// acc += sum over the entries j0 <= j < j1 of the chunk of val[j] * B[col[j], this lane's chunk).
// j0, j1 are the same in all lanes: the (column, value) pair of entry j is read out of lane j into
// scalar registers, D rows of B are in flight, and the last 1..D-1 entries go as one more round in
// which the missing ones load nothing and add +0.  (A lane whose chunk of columns would lie past the
// last column is given a chunk that exists and its sums are thrown away by the caller: a load that
// shares its cache line with a neighbour's costs less than the branches that would mask it.)
template <int VEC, bool OFF32, int D>
__device__ __forceinline__ void chunk_accumulate(const UniformRows<VEC, OFF32>& rows, Vec<VEC>& acc,
                                                 const EntryChunk& ch, int j0, int j1)
{
    int j = j0;
    for (; j + D <= j1; j += D) {
        int32_t c[D];
        float v[D];
        Vec<VEC> b[D];
#pragma unroll
        for (int u = 0; u < D; ++u) {
            c[u] = __builtin_amdgcn_readlane(ch.col, j + u);
            v[u] = __int_as_float(__builtin_amdgcn_readlane(ch.val, j + u));
        }
#pragma unroll
        for (int u = 0; u < D; ++u) b[u] = rows.load(c[u]);
#pragma unroll
        for (int u = 0; u < D; ++u) acc.fma(v[u], b[u]);
    }
    if (j < j1) {
        const int rem = j1 - j;
        int32_t c[D - 1];
        float v[D - 1];
        Vec<VEC> b[D - 1];
#pragma unroll
        for (int u = 0; u < D - 1; ++u) {
            // (lane j + u exists for every u: j < 64 and the lane number wraps at 64)
            c[u] = __builtin_amdgcn_readlane(ch.col, (j + u) & (kWave - 1));
            v[u] = u < rem ? __int_as_float(__builtin_amdgcn_readlane(ch.val, (j + u) & (kWave - 1))) : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < D - 1; ++u) {
            b[u].zero();
            if (u < rem) b[u] = rows.load(c[u]);
        }
#pragma unroll
        for (int u = 0; u < D - 1; ++u) acc.fma(v[u], b[u]);
    }
}

}  // namespace sgap
