// The gather-multiply-accumulate inner loop shared by the schedules: stored
// entries come from an LDS copy of colidx/vals, rows of B from memory.
#pragma once
#include "sgap_common.hpp"

namespace sgap {

// LDS copy of one stored entry of A
struct StagedEntry {
    int32_t col;
    float val;
};

// Coalesced streaming copy of stored entries [base, base+cnt) into LDS.
// The caller synchronises.
__device__ __forceinline__ void stage_entries(const SpmmArgs& a, uint32_t base, uint32_t cnt,
                                              StagedEntry* __restrict__ s_A, uint32_t block = kBlock)
{
    for (uint32_t q = threadIdx.x; q < cnt; q += block) {
        StagedEntry e;
        e.col = load_stream(a.colidx + base + q);
        e.val = load_stream(a.vals + base + q);
        s_A[q] = e;
    }
}

// Where the rows of B come from: the `col` field of a staged entry is the key
// handed to load().
template <int VEC, bool OFF32>
struct GlobalRows {
    BRow<OFF32> b;
    __device__ __forceinline__ GlobalRows(const float* B, int64_t n, int64_t k) : b(B, n, k) {}
    __device__ __forceinline__ Vec<VEC> load(int32_t col) const { return load_vec<VEC>(b.at(col)); }
};

// U entries q, q+STRIDE, ... : all U rows of B are requested before the first
// is consumed.
template <int VEC, int STRIDE, int U, typename SRC>
__device__ __forceinline__ void gather_batch(Vec<VEC>& acc, const StagedEntry* __restrict__ s_A, uint32_t q,
                                             const SRC& B)
{
    StagedEntry e[U];
    Vec<VEC> b[U];
#pragma unroll
    for (int j = 0; j < U; ++j) e[j] = s_A[q + j * STRIDE];
#pragma unroll
    for (int j = 0; j < U; ++j) b[j] = B.load(e[j].col);
#pragma unroll
    for (int j = 0; j < U; ++j) acc.fma(e[j].val, b[j]);
}

// The last 1..U entries q, q+STRIDE, ... < q1 as one batch: entries past q1
// load nothing and contribute +0.
template <int VEC, int STRIDE, int U, typename SRC>
__device__ __forceinline__ void gather_tail(Vec<VEC>& acc, const StagedEntry* __restrict__ s_A, uint32_t q,
                                            uint32_t q1, const SRC& B)
{
    StagedEntry e[U];
    Vec<VEC> b[U];
#pragma unroll
    for (int j = 0; j < U; ++j) {
        e[j].col = 0;
        e[j].val = 0.0f;
        if (q + j * STRIDE < q1) e[j] = s_A[q + j * STRIDE];
    }
#pragma unroll
    for (int j = 0; j < U; ++j) {
        b[j].zero();
        if (q + j * STRIDE < q1) b[j] = B.load(e[j].col);
    }
#pragma unroll
    for (int j = 0; j < U; ++j) acc.fma(e[j].val, b[j]);
}

// Gathered rows of B a lane keeps in flight.  Six, not eight: the row-split
// kernel then needs 78 instead of 90 vector registers and a SIMD holds six
// wavefronts instead of five, which is worth more on the 27-entry rows of the
// stencil workload (0.66 -> 0.615 ms) than the deeper batch.
constexpr int kGatherDepth = 6;

// acc += sum over LDS slots q = q0, q0+STRIDE, ... < q1 of val[q] * B[col[q], k..k+VEC)
// Full batches of kGatherDepth, then the remaining entries as one more round
// of predicated loads, so that a row costs ceil(len/kGatherDepth) memory round
// trips.
template <int VEC, int STRIDE, typename SRC>
__device__ __forceinline__ void gather_fma(Vec<VEC>& acc, const StagedEntry* __restrict__ s_A, uint32_t q0,
                                           uint32_t q1, const SRC& B)
{
    constexpr int D = kGatherDepth;
    uint32_t q = q0;
    for (; q + (D - 1) * STRIDE < q1; q += D * STRIDE) gather_batch<VEC, STRIDE, D>(acc, s_A, q, B);
    if (q >= q1) return;
    if (q + (D / 2) * STRIDE < q1) gather_tail<VEC, STRIDE, D>(acc, s_A, q, q1, B);
    else gather_tail<VEC, STRIDE, D / 2>(acc, s_A, q, q1, B);
}

}  // namespace sgap
