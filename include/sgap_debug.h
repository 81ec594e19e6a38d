/*
 * sgap_debug.h - test and measurement scaffolding of the MI355X CSR SpMM
 * library: exported by the same shared library as sgap.h's calls, but not
 * part of the interface an application programs against.  Used by the parity
 * tests (device self-checks of the cross-lane primitives, host-side pieces of
 * the schedules) and by the benchmark (event timing of the library's own
 * launches, a streaming copy that the hardware counters are calibrated on).
 * Conventions as in sgap.h.
 */
#ifndef SGAP_DEBUG_H
#define SGAP_DEBUG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Timing hooks for benchmarks.  While enabled, every compute call (SpMM,
 * SDDMM, TTM, MTTKRP) brackets ALL the kernels it enqueues (the row-zeroing
 * pass and the preparation of the window path included) with a pair of HIP
 * events on the call's stream.  sgap_profile_collect waits for those events,
 * adds their elapsed times in milliseconds into *total_ms, their number into
 * *count, and forgets them.  Not thread-safe; host pointers.
 */
int sgap_profile_enable(int on);
int sgap_profile_collect(double* total_ms, int* count);

/*
 * Device self-checks of the two cross-lane primitives behind the strategies
 * (the paper's macro instructions atomicAddGroup<T,G> and
 * segReduceGroup<T,G>, Section 5.3), one wavefront each.  `lanes_per_row`
 * (1..64/group_size, power of two) is the lane stride between neighbouring
 * members of a group.
 *   sgap_debug_group_reduce: in fp32[64] device -> out fp32[64] device; the
 *     first lane of every group receives the sum of its group's inputs, other
 *     lanes receive 0.
 *   sgap_debug_group_seg_reduce: in fp32[64], span int32[64] device (span[l] =
 *     how many following members of lane l's group continue lane l's run,
 *     0..group_size-1) -> out[l] = in[l] + the next span[l] members' inputs.
 *   sgap_debug_group_partial_reduce: the same for sub-groups of reduce_size
 *     members (power of two <= group_size): the first lane of every sub-group
 *     receives the sub-group's sum, other lanes 0.
 */
int sgap_debug_group_reduce(const float* in, float* out, int group_size,
                            int lanes_per_row, void* stream);
int sgap_debug_group_partial_reduce(const float* in, float* out, int group_size,
                                    int reduce_size, int lanes_per_row, void* stream);
int sgap_debug_group_seg_reduce(const float* in, const int32_t* span, float* out,
                                int group_size, int lanes_per_row, void* stream);

/*
 * Host-side pieces of the nnz-balanced schedule, exported for tests; no GPU
 * is touched.
 *   sgap_debug_tile_deal: which tiles of stored entries workgroup `block` of a
 *     persistent grid of `grid` workgroups takes when the matrix has `tiles`
 *     tiles (chunks of neighbouring tiles per die).  Writes up to `capacity`
 *     tile numbers, ascending, into out_tiles (host) and returns how many
 *     tiles the workgroup takes, or -1 on bad arguments.
 *   sgap_debug_plan_nnz_serial: tile size (stored entries), whether a
 *     tile's partial sums are merged on chip, and the chunk lanes per stored
 *     entry the kernel runs with (lanes_per_row, or fewer where the on-chip
 *     accumulators of a small group would not fit otherwise), for the serial
 *     strategy with lanes_per_row chunk lanes of cols_per_lane columns each on
 *     a chip of compute_units; forced_tile as sgap_config.nnz_tile.  Host
 *     pointers; lanes_used may be null.
 */
int64_t sgap_debug_tile_deal(int64_t tiles, int grid, int block, int64_t* out_tiles, int64_t capacity);
int sgap_debug_plan_nnz_serial(int group_size, int lanes_per_row, int cols_per_lane, int64_t nnz_hint,
                               int compute_units, int forced_tile, int* tile, int* merge_on_chip,
                               int* lanes_used);

/*
 * Streaming kernels over n fp32 elements (16-byte aligned device buffers):
 * what the memory system delivers to a kernel that does nothing but stream,
 * reported next to the roofline fractions, and what the hardware traffic
 * counters are calibrated on.
 *   mode 0  copy src -> dst (sgap_copy_f32 is this)
 *   mode 1  read src only; dst points to one float that is (in practice
 *           never) written, so that the reads cannot be optimised away
 *   mode 2  write dst only (the value 1.0f); src is ignored
 */
int sgap_stream_f32(const float* src, float* dst, int64_t n, int mode, void* stream);
int sgap_copy_f32(const float* src, float* dst, int64_t n, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SGAP_DEBUG_H */
