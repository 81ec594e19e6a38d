// Row-split schedule, serial strategy, with the widest lane layout: the point
// {<g row, c col>, 1} of the paper's design space (Section 6.1) with all 64
// lanes of a wavefront on neighbouring column chunks (LC = 64, c = VEC columns
// per lane), so that one wavefront owns g consecutive rows of A and one column
// tile of 64*VEC columns of B and C.  Every lane of the wavefront then wants the
// same stored entry (sgap_uniform.hpp): per stored entry the kernel issues two
// lane reads, one scalar multiply, one buffer load and VEC multiply-adds, needs
// no LDS and few vector registers, and a compute unit holds the most wavefronts
// the hardware allows.
//
// The stored entries of a wavefront's rows are contiguous in colidx/vals, so the
// wavefront walks them in aligned runs of 64 (one coalesced load, the next run
// requested a run ahead) and D at a time without regard to row ends: D rows of
// B are in flight whatever the row lengths are, and a row that ends inside a
// batch is stored (plain streaming store, one owner per row: no atomics, empty
// rows get zeros) before the next entry is added.
#include "sgap_common.hpp"
#include "sgap_uniform.hpp"

namespace sgap {

constexpr int kWaveRowsMax = 63;  // rows per wavefront at most: their rowptr slice sits in one vector register

template <int VEC, bool OFF32, int D, bool SKIP>
__global__ __launch_bounds__(kBlock) void wave_rows_kernel(const int32_t* __restrict__ rowptr,
                                                           const int32_t* __restrict__ colidx,
                                                           const float* __restrict__ vals, const float* __restrict__ B,
                                                           float* __restrict__ C, int64_t M, int64_t K, int64_t N,
                                                           TileSched ts, int rows_per_wave, RowSkip skip)
{
    const int lane = threadIdx.x % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    bool skip_on = false;
    if constexpr (SKIP) skip_on = *skip.count <= skip.max_rows;

    // work item of this workgroup: (block of 4 * rows_per_wave rows, tile of 64 * VEC columns), with every die
    // taking one contiguous run of the column-tile-major item order (see TileSched)
    const int64_t item = (int64_t)(blockIdx.x % ts.xcds) * ts.items_per_xcd + blockIdx.x / ts.xcds;
    if (item >= ts.items) return;
    const int32_t col_tile = (int32_t)(item / ts.row_blocks);
    const int64_t row_block = item % ts.row_blocks;
    const int64_t row0 = (row_block * kWavesPerBlock + wave) * rows_per_wave;
    if (row0 >= M) return;
    const int nrows = (int)(M - row0 < rows_per_wave ? M - row0 : rows_per_wave);

    const int64_t k = (int64_t)col_tile * (kWave * VEC) + lane * VEC;
    const bool k_ok = k < N;
    const UniformRows<VEC, OFF32> rows(B, K, N, k_ok ? k : 0);

    // lane i holds rowptr[row0 + i], i <= nrows
    // (every lane stays active to the end: the values of rp are read across lanes below, and a lane that had
    // left would not hold its value.  Lanes past the last column work on the first chunk and store nothing.)
    const int32_t rp = rowptr[row0 + (lane <= nrows ? lane : nrows)];
    const int32_t pend = __builtin_amdgcn_readlane(rp, nrows);
    int32_t p = __builtin_amdgcn_readlane(rp, 0);
    int row = -1;          // no row yet; the first pass of the loop below enters row 0
    int32_t row_end = p;
    bool skipped = true;   // nothing to store for "row -1"
    Vec<VEC> acc;
    acc.zero();
    // the run of 64 entries that holds position p, and the run after it
    int32_t run = p & ~(kWave - 1);
    EntryChunk cur = load_chunk(colidx, vals, run, pend, lane);
    EntryChunk ahead = load_chunk(colidx, vals, run + kWave, pend, lane);

    auto finish_row = [&]() {
        if (!skipped && k_ok) store_vec_stream<VEC>(C + (row0 + row) * N + k, acc);
        acc.zero();
    };

    for (;;) {
        // finish the rows that end at p and enter the row that holds position p
        bool done = false;
        while (p >= row_end) {
            finish_row();
            if (++row >= nrows) {
                done = true;
                break;
            }
            row_end = __builtin_amdgcn_readlane(rp, row + 1);
            skipped = false;
            if constexpr (SKIP) {
                skipped = skip_on && row_end - p >= skip.min_len;  // p is the row's first position here
                if (skipped) p = row_end;
            }
        }
        if (done) break;
        if (p >= run + kWave) {
            // on to the next run (or, past a row that was left out, to the run that holds p)
            if (p < run + 2 * kWave) {
                cur = ahead;
                run += kWave;
            } else {
                run = p & ~(kWave - 1);
                cur = load_chunk(colidx, vals, run, pend, lane);
            }
            ahead = load_chunk(colidx, vals, run + kWave, pend, lane);
        }

        // one batch: the entries p .. p + cnt - 1 of the run, whatever rows they belong to
        const int j = p - run;
        int cnt = pend - p < D ? pend - p : D;
        if (kWave - j < cnt) cnt = kWave - j;
        int32_t c[D];
        float v[D];
        Vec<VEC> b[D];
#pragma unroll
        for (int u = 0; u < D; ++u) {
            c[u] = __builtin_amdgcn_readlane(cur.col, (j + u) & (kWave - 1));
            v[u] = __int_as_float(__builtin_amdgcn_readlane(cur.val, (j + u) & (kWave - 1)));
        }
        if (cnt == D) {
#pragma unroll
            for (int u = 0; u < D; ++u) b[u] = rows.load(c[u]);
        } else {
#pragma unroll
            for (int u = 0; u < D; ++u) {
                b[u].zero();
                if (u < cnt) b[u] = rows.load(c[u]);
            }
        }
        int32_t next_p = p + cnt;
        bool live = true;  // false once the batch has run into a row that is left out
#pragma unroll
        for (int u = 0; u < D; ++u) {
            if (!live || u >= cnt) continue;
            if (p + u >= row_end) {
                // entry p + u opens another row (row < nrows - 1 here, because p + u < pend)
                do {
                    finish_row();
                    ++row;
                    row_end = __builtin_amdgcn_readlane(rp, row + 1);
                    skipped = false;
                } while (p + u >= row_end);
                if constexpr (SKIP) {
                    skipped = skip_on && row_end - (p + u) >= skip.min_len;
                    if (skipped) {
                        next_p = row_end;  // the rest of the batch belongs to a row another kernel produces
                        live = false;
                        continue;
                    }
                }
            }
            acc.fma(v[u], b[u]);
        }
        p = next_p;
    }
}

namespace {

template <int VEC, int D>
hipError_t launch_wave_rows_vec(const SpmmArgs& a, int rows_per_wave, int xcds, const RowSkip* skip, hipStream_t s)
{
    TileSched ts;
    const int64_t rows_per_block = (int64_t)kWavesPerBlock * rows_per_wave;
    ts.row_blocks = (a.M + rows_per_block - 1) / rows_per_block;
    ts.tile_cols = kWave * VEC;
    ts.col_tiles = (int32_t)((a.N + ts.tile_cols - 1) / ts.tile_cols);
    ts.items = ts.row_blocks * ts.col_tiles;
    ts.xcds = xcds;
    ts.items_per_xcd = (ts.items + xcds - 1) / xcds;
    if (ts.items_per_xcd * xcds > 0x7ffffff0LL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(ts.items_per_xcd * xcds)), block(kBlock);
    const bool off32 = offsets_fit_32(a);
    const RowSkip none{nullptr, 0, 0};
    if (skip) {
        if (off32)
            hipLaunchKernelGGL((wave_rows_kernel<VEC, true, D, true>), grid, block, 0, s, a.rowptr, a.colidx, a.vals, a.B,
                               a.C, a.M, a.K, a.N, ts, rows_per_wave, *skip);
        else
            hipLaunchKernelGGL((wave_rows_kernel<VEC, false, D, true>), grid, block, 0, s, a.rowptr, a.colidx, a.vals, a.B,
                               a.C, a.M, a.K, a.N, ts, rows_per_wave, *skip);
    } else {
        if (off32)
            hipLaunchKernelGGL((wave_rows_kernel<VEC, true, D, false>), grid, block, 0, s, a.rowptr, a.colidx, a.vals,
                               a.B, a.C, a.M, a.K, a.N, ts, rows_per_wave, none);
        else
            hipLaunchKernelGGL((wave_rows_kernel<VEC, false, D, false>), grid, block, 0, s, a.rowptr, a.colidx, a.vals,
                               a.B, a.C, a.M, a.K, a.N, ts, rows_per_wave, none);
    }
    return hipGetLastError();
}

}  // namespace

// vec = columns per lane (1, 2 or 4; N % vec == 0 and B, C aligned to vec * 4 bytes), rows_per_wave in
// 1..kWaveRowsMax, skip = rows another kernel produces (or nullptr)
hipError_t launch_wave_rows(const SpmmArgs& a, int vec, int rows_per_wave, int xcds, const RowSkip* skip,
                            hipStream_t s)
{
    if (rows_per_wave < 1 || rows_per_wave > kWaveRowsMax || xcds < 1) return hipErrorInvalidValue;
    switch (vec) {
        case 4: return launch_wave_rows_vec<4, 8>(a, rows_per_wave, xcds, skip, s);
        case 2: return launch_wave_rows_vec<2, 8>(a, rows_per_wave, xcds, skip, s);
        case 1: return launch_wave_rows_vec<1, 8>(a, rows_per_wave, xcds, skip, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sgap
