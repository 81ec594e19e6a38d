/*
 * sgap.h - C ABI of the MI355X (gfx950) CSR SpMM library.
 *
 *   C[M,N] = A_csr[M,K] * B[K,N]      fp32, A in CSR, B and C dense row-major
 *
 * The operation is the SpMM form of the paper's sparse-dense hybrid algebra
 * (Section 2.1, last of the forms listed under Eq. 1).  How the sum over a
 * row's stored entries is organised follows the paper's "atomic parallelism"
 * design space (Section 3) through the "segment group" abstraction
 * (Section 4): a group of `group_size` lanes is the unit of synchronisation,
 * and `strategy` says how a group turns per-lane products into row sums.
 * Every (group_size, strategy, schedule) point computes the same C; only the
 * order of fp32 additions differs.
 *
 * Conventions for every entry point
 *   - All array arguments are DEVICE pointers owned by the caller.  The
 *     library reads rowptr/colidx/vals/B, overwrites C, keeps no pointer
 *     after the call returns and allocates no device memory.  The one path
 *     that needs working memory (long rows by column windows, see
 *     sgap_spmm_csr_cfg) takes it from the caller, who may use it for
 *     something else once the work enqueued by the call has finished; calls
 *     that are given different workspaces may run concurrently on different
 *     streams.  (sgap_validate_csr keeps four counters in a file-scope device
 *     array of the library, one copy per GPU: calls to it must not overlap on
 *     one GPU.)
 *   - The library keeps a little host-side state without locks (the schedule
 *     and tuning defaults, cached device properties, the profiling event
 *     list): call it from one host thread at a time; any number of streams.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and the call returns without waiting.
 *   - A call only enqueues kernels (no allocation, no host synchronisation, no
 *     memset nodes), so it may be recorded into a HIP graph; the first call
 *     that uses a kernel instance asks the runtime for its occupancy and
 *     should be made once outside a capture.
 *   - Return value: an sgap_status.  SGAP_ERR_INVALID_ARG and
 *     SGAP_ERR_UNSUPPORTED are found before anything is launched and leave C
 *     untouched; after SGAP_ERR_HIP (the runtime refused a launch) some of the
 *     call's kernels may already be enqueued and the contents of C are
 *     undefined.  sgap_last_error() gives detail.
 *   - Preconditions that are NOT checked on the device: rowptr[0] == 0,
 *     rowptr non-decreasing, rowptr[M] == number of stored entries,
 *     0 <= colidx[p] < K.  Column indices inside a row need not be sorted
 *     or distinct (duplicates add).  Explicit zeros are ordinary entries.
 *   - Indices are 0-based int32; element offsets are formed in 64 bits.
 *     Positions of stored entries are 32-bit: rowptr[M] may be at most
 *     2^31 - 65,536 (2,147,418,112; a hint beyond that is refused), which
 *     leaves room for the kernels to step past the end by a tile.
 *   - Semantics are OVERWRITE (C = A*B): rows without stored entries become
 *     +0, whatever C held before.  A row's result may be -0 or +0 where the
 *     exact sum is zero.
 *   - Placement (speed only, never results): any 4-byte aligned addresses are
 *     accepted (16-byte aligned B and C allow 16-byte loads).  Where rows of B
 *     are gathered at random out of memory, the operands of one matrix are
 *     served faster out of ONE allocation, packed one after the other, than
 *     out of five allocations that each start on a large page boundary
 *     (R-MAT with 2^21 rows and 50 M entries, N = 32: 0.70 against 0.86 ms for
 *     the same bytes moved).
 */
#ifndef SGAP_H
#define SGAP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SGAP_OK = 0,
    SGAP_ERR_INVALID_ARG = 1, /* bad size, enum, group size or null pointer   */
    SGAP_ERR_UNSUPPORTED = 2, /* valid request this build cannot serve        */
    SGAP_ERR_HIP = 3          /* the HIP runtime reported an error on launch  */
} sgap_status;

/*
 * Reduction strategy of a segment group (Section 4.2 "ReductionStrategy";
 * the parallel / serial axis of Section 3.3's mapping to earlier SpMM
 * algorithm spaces).
 *
 * SGAP_REDUCE_PARALLEL: group_size lanes of one wavefront each take a share
 *   of the stored entries and combine their partial sums with cross-lane
 *   operations.
 *     row-split schedule   : the group_size lanes share one row
 *       ({<1/g row, c col>, r} with g = r = group_size, Section 6.2); a plain
 *       tree sum, one writeback lane, plain store.
 *     nnz-balanced schedule: lane = one stored entry ({<1 nnz, c col>, r},
 *       Section 6.2); the group performs a SEGMENTED reduction keyed by row
 *       (Fig. 1c), one writeback lane per run of equal rows.
 * SGAP_REDUCE_SERIAL: reduction parallelism 1.  Each lane walks group_size
 *   consecutive units by itself and flushes its register when the row changes
 *   ("conditional" reduction).
 *     row-split schedule   : lane = group_size consecutive rows
 *       ({<g row, c col>, 1}, Section 6.1), plain stores.
 *     nnz-balanced schedule: lane = group_size consecutive stored entries
 *       ({<g nnz, c col>, 1}, Section 6.1).
 *
 * In the nnz-balanced schedule a row whose stored entries all lie inside one
 * aligned block of positions (group_size positions, or a whole tile of about a
 * thousand when the partial sums of a tile fit on chip) is written with one
 * plain store; only a row that crosses such a block is zeroed first and
 * receives its partial sums by atomic adds.
 */
typedef enum { SGAP_REDUCE_PARALLEL = 0, SGAP_REDUCE_SERIAL = 1 } sgap_strategy;

/*
 * Work partition (Section 3.2: minimal data counted in rows or in non-zeros).
 * SGAP_SCHED_ROW_SPLIT   : units of work are rows of A.
 * SGAP_SCHED_NNZ_BALANCED: units of work are equal runs of stored entries;
 *   the row of an entry is found by searching rowptr (Listings 1 and 2).
 */
typedef enum { SGAP_SCHED_ROW_SPLIT = 0, SGAP_SCHED_NNZ_BALANCED = 1 } sgap_schedule;

/* Process-wide schedule used by sgap_spmm_csr(); default SGAP_SCHED_ROW_SPLIT.
 * sgap_set_schedule returns SGAP_ERR_INVALID_ARG for an unknown value. */
int sgap_set_schedule(int schedule);
int sgap_get_schedule(void);

/*
 * C = A*B with the process-wide schedule.
 *   M, K, N     rows of A and C; columns of A = rows of B; columns of B and C.
 *               All >= 0, M <= 2^31-2, N < 2^31.  M == 0 or N == 0: SGAP_OK,
 *               nothing to do.
 *   rowptr      device, int32[M+1]
 *   colidx      device, int32[rowptr[M]]   (may be NULL only if A is known
 *               empty, i.e. never dereferenced when rowptr[M] == 0)
 *   vals        device, fp32[rowptr[M]]
 *   B           device, fp32[K*N], row-major, leading dimension N
 *   C           device, fp32[M*N], row-major, leading dimension N; overwritten
 *   group_size  1, 2, 4, 8, 16, 32 or 64 (lanes of a wave64 segment group for
 *               SGAP_REDUCE_PARALLEL; units per lane for SGAP_REDUCE_SERIAL)
 *   strategy    an sgap_strategy
 *   stream      hipStream_t or NULL
 * The number of dense columns per lane (the paper's c) is chosen from N and
 * the pointer alignment: 4 (one 16-byte load) if N % 4 == 0 and B, C are
 * 16-byte aligned, else 2, else 1 (Section 7.2, coarsening rule).
 * The nnz-balanced schedule reads rowptr[M] on the device and runs a
 * fixed-size grid, so this call never synchronises with the host.
 */
int sgap_spmm_csr(int64_t M, int64_t K, int64_t N,
                  const int32_t* rowptr, const int32_t* colidx, const float* vals,
                  const float* B, float* C,
                  int group_size, int strategy, void* stream);

/*
 * Same, with the schedule passed explicitly (no process-wide state) and an
 * optional host-side count of stored entries.
 *   schedule    an sgap_schedule
 *   nnz_hint    rowptr[M] if the caller knows it, else -1.  Only used to size
 *               the nnz-balanced grid (a hint larger than the truth is safe;
 *               a smaller one is also safe, only slower).
 */
int sgap_spmm_csr_ex(int64_t M, int64_t K, int64_t N,
                     const int32_t* rowptr, const int32_t* colidx, const float* vals,
                     const float* B, float* C,
                     int group_size, int strategy, int schedule,
                     int64_t nnz_hint, void* stream);

/*
 * Row-split SpMM with the tiling and the synchronisation granularity set
 * apart: the point {<1/g row, c col>, r} of the paper's design space
 * (Section 4; Table 1 sweeps r below g).  `group_size` = g lanes share a row
 * and split its stored entries; every `reduce_size` = r neighbouring lanes of
 * them (power of two, 1 <= r <= g) tree-sum their partial sums, and the g/r
 * sub-group sums of a row are merged into C with atomic adds (r = 1: every
 * lane adds its own sum: the group is parallelised with the "Atomics" output
 * strategy alone, as in the schedule printed in Section 6.2).  r = g is
 * sgap_spmm_csr_ex with the parallel strategy and the row-split schedule:
 * plain stores, no atomics.  For r < g the library zeroes C first, and the
 * order of the atomic adds, hence the fp32 rounding, varies between runs.
 * Other arguments, ownership and errors as for sgap_spmm_csr_ex.
 */
int sgap_spmm_csr_gr(int64_t M, int64_t K, int64_t N,
                     const int32_t* rowptr, const int32_t* colidx, const float* vals,
                     const float* B, float* C,
                     int group_size, int reduce_size, int64_t nnz_hint, void* stream);

/*
 * Per-call configuration: the point of the design space (schedule, strategy,
 * group_size, reduce_size as for the calls above) together with the tiling
 * parameters that the paper tunes apart from the synchronisation granularity
 * (Section 7.2: the space <groupSz, blockSz, tileSz, workerDimR> of Tables 4
 * and 5; here group_size, block_size, tile_cols and rows_per_group).  Zero
 * (-1 for xcd_remap) leaves a choice to the library.  None of them changes the
 * result beyond the order of fp32 additions.
 *   reduce_size     0 or group_size: the whole group reduces; a smaller power
 *                   of two: sub-groups merged with atomics (row-split schedule,
 *                   parallel strategy only; see sgap_spmm_csr_gr).
 *   block_size      threads per workgroup of the row-split schedule: 128, 256
 *                   or 512 (automatic: 256).  block_size / (lanes per row x
 *                   lanes per column tile) groups work side by side on
 *                   neighbouring rows.
 *   tile_cols       columns of B/C per work item of the row-split schedule
 *                   (rounded up to the vector width, capped at N; automatic:
 *                   128); with the vector width it fixes the lanes that share
 *                   a row of B, hence how many rows a workgroup works on at once.
 *   rows_per_group  rows one group works through per work item in the row-split
 *                   parallel strategy (the serial strategy takes group_size rows
 *                   by definition); automatic: from the mean row length.
 *   xcd_remap       1/-1: hand each of the 8 dies a contiguous run of work items
 *                   so that its L2 keeps the rows of B it gathers; 0: plain
 *                   round-robin order.
 *   persistent      1: the row-split schedule launches only as many workgroups
 *                   as the chip holds at once and each loops over work items.
 *   nnz_tile        stored entries per tile of the nnz-balanced serial strategy:
 *                   256, 512, 1024 or 2048 (the two small ones need N % 4 == 0
 *                   and 16-byte aligned B and C, else the automatic choice is kept).
 *   wave_rows       lane layout of the row-split serial strategy: 1 = one wavefront
 *                   owns group_size consecutive rows (at most 63) and all its 64
 *                   lanes hold column chunks of c = 4, 2 or 1 columns, so that a
 *                   stored entry is the same for the whole wavefront ({<g row,
 *                   c col>, 1} of Section 6.1 with the widest lane layout; from 48
 *                   columns on); -1 = never; 0 = automatic: only for the rows that
 *                   long_row_min leaves to the row-split kernel, from 192 columns on.
 *   long_row_min    row-split schedule, reduce_size = group_size, N % 4 == 0 and
 *                   16-byte aligned B and C only (ignored otherwise): rows of at
 *                   least this many stored entries (say 1024) are taken out of the
 *                   row-split kernel and produced by column windows: the columns
 *                   are cut into windows of window_kb KiB of B, a die works on one
 *                   window at a time so that its L2 serves the gathers, and the
 *                   pieces of a long row are added into C with atomic adds (the
 *                   "Atomics" output strategy of Section 6.2; fp32 rounding then
 *                   varies between runs, as on the nnz-balanced schedule).  Worth
 *                   it when long rows hold most entries and B is far larger than
 *                   the L2s.  Needs a workspace (below).  0 = off.
 *   window_kb       KiB of B per column window (at most 511 windows are made);
 *                   automatic: 3072.
 *   max_long_rows   capacity of the list of long rows, at most 1,048,576;
 *                   automatic: 8192.  The rows are found on the device; when a
 *                   matrix has more long rows than this, the call produces every
 *                   row with the row-split kernel instead (correct, slower).
 */
typedef struct {
    int schedule;
    int strategy;
    int group_size;
    int reduce_size;
    int block_size;
    int tile_cols;
    int rows_per_group;
    int xcd_remap;
    int persistent;
    int nnz_tile;
    int wave_rows;
    int long_row_min;
    int window_kb;
    int max_long_rows;
} sgap_config;

/* Fill *config with the defaults: row-split schedule, parallel strategy, group
 * size 8, every tiling choice left to the library, long rows not set apart. */
int sgap_config_init(sgap_config* config);

/*
 * Bytes of device workspace that sgap_spmm_csr_cfg needs for this shape and
 * configuration: 0 when long_row_min is 0 (or the window path cannot apply:
 * another schedule, reduce_size < group_size, N % 4 != 0), else a 256-byte
 * header plus 4 * max_long_rows * (windows + 3) bytes, where windows =
 * ceil(K / rows of B per window).  Returns -1 for invalid arguments.
 */
int64_t sgap_spmm_csr_workspace_size(int64_t M, int64_t K, int64_t N, const sgap_config* config);

/*
 * C = A*B at the point and with the tiling that *config names (host pointer,
 * read during the call only).  Arguments, ownership and errors as for
 * sgap_spmm_csr_ex, and:
 *   workspace        device memory, 256-byte aligned, at least
 *                    sgap_spmm_csr_workspace_size(M, K, N, config) bytes; may be
 *                    NULL when that is 0.  The call's kernels write and read it;
 *                    its contents afterwards mean nothing to the caller.  Two
 *                    calls that may run at the same time need two workspaces.
 *   workspace_bytes  its size; a size below the need is SGAP_ERR_INVALID_ARG.
 * The call only enqueues kernels on `stream`: no allocation, no host
 * synchronisation, no memset node.
 */
int sgap_spmm_csr_cfg(int64_t M, int64_t K, int64_t N,
                      const int32_t* rowptr, const int32_t* colidx, const float* vals,
                      const float* B, float* C,
                      const sgap_config* config, int64_t nnz_hint,
                      void* workspace, int64_t workspace_bytes, void* stream);

/*
 * sgap_spmm_csr_cfg for callers that cannot allocate device memory, not even
 * for a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  The same call with the working memory of the window
 * path in an array of 8 MiB (8,388,608 bytes) that the library holds on every
 * GPU it runs on until the process ends; no workspace arguments, and neither
 * this call nor anything it calls allocates or frees (no hipMalloc, no
 * hipFree, no allocating library routine).  The caller still passes operands
 * and result.
 *   - A shape and configuration whose sgap_spmm_csr_workspace_size exceeds
 *     8,388,608 bytes is refused with SGAP_ERR_UNSUPPORTED before anything is
 *     launched (say, more windows or a longer list than fit: lower
 *     max_long_rows or raise window_kb), with the two sizes in
 *     sgap_last_error().  A configuration that needs no working memory runs as
 *     sgap_spmm_csr_cfg does.
 *   - Every call on a GPU uses that GPU's one array, which keeps the last
 *     call's contents; the call resets what it reads before writing.  Calls
 *     that may overlap in time on one GPU (two streams, two threads) race on
 *     it: the caller must order them.  sgap_spmm_csr_cfg with two workspaces
 *     is the entry point for overlapping calls.
 *   - The first call on a device looks up the array's device address
 *     (hipGetSymbolAddress, with that device current); make it outside a
 *     graph capture.
 * Results, other arguments and errors as for sgap_spmm_csr_cfg.
 */
int sgap_spmm_csr_cfg_static(int64_t M, int64_t K, int64_t N,
                             const int32_t* rowptr, const int32_t* colidx, const float* vals,
                             const float* B, float* C,
                             const sgap_config* config, int64_t nnz_hint, void* stream);

/*
 * Sampled dense-dense matrix product on the pattern of a CSR matrix, the
 * SDDMM form of the paper's Section 2.1 (third form under Eq. 1):
 *   out_vals[p] = vals[p] * sum_{j<J} X1[row(p), j] * X2T[colidx[p], j]
 * for every stored entry p of A (M x K, CSR as for sgap_spmm_csr; row(p) is
 * the row whose rowptr range holds p).  The paper names it next to SpMM
 * because its reduction, here along the dense dimension j, is served by the
 * same segment-group reductions.
 *   X1        device, M x J row-major, ld = J
 *   X2T       device, K x J row-major, ld = J: the second dense operand
 *             transposed, X2T[k, j] = X2[j, k], so that both factors of an
 *             entry are contiguous rows
 *   out_vals  device, rowptr[M] values in the order of colidx; OVERWRITTEN.
 *             May not alias vals.
 *   group_size, strategy
 *             SGAP_REDUCE_PARALLEL: group_size lanes share a stored entry,
 *             split j between them and tree-sum; SGAP_REDUCE_SERIAL: every
 *             lane computes group_size consecutive stored entries by itself.
 *   nnz_hint  rowptr[M] if the host knows it, else -1 (sizes the grid; 0
 *             returns at once).
 * Every output has one writer: no atomics, results are reproducible run to
 * run.  Asynchronous on `stream`; ownership and errors as for sgap_spmm_csr.
 * J == 0 writes zeros.  colidx, vals and out_vals may be null only for a
 * matrix without stored entries.
 */
int sgap_sddmm_csr(int64_t M, int64_t K, int64_t J,
                   const int32_t* rowptr, const int32_t* colidx, const float* vals,
                   const float* X1, const float* X2T, float* out_vals,
                   int group_size, int strategy, int64_t nnz_hint, void* stream);

/*
 * The same product with the stored entries of long rows taken by column
 * windows of X2T, as sgap_spmm_csr_cfg does for SpMM (same reasoning: a die
 * works on one window at a time so that its L2 serves the gathered rows of
 * X2T).  Applies when J % 4 == 0, 32 <= J <= 256 and X1, X2T are 16-byte
 * aligned; otherwise the call is sgap_sddmm_csr.  Every entry still has one
 * writer: no atomics, results reproducible.
 *   long_row_min, window_kb (automatic: 2048), max_long_rows
 *                    as in sgap_config
 *   workspace, workspace_bytes
 *                    device memory, 256-byte aligned, of at least
 *                    sgap_sddmm_csr_workspace_size(K, J, window_kb,
 *                    max_long_rows) bytes (0: the path does not apply; -1:
 *                    invalid arguments)
 */
int sgap_sddmm_csr_windows(int64_t M, int64_t K, int64_t J,
                           const int32_t* rowptr, const int32_t* colidx, const float* vals,
                           const float* X1, const float* X2T, float* out_vals,
                           int group_size, int strategy, int64_t nnz_hint,
                           int long_row_min, int window_kb, int max_long_rows,
                           void* workspace, int64_t workspace_bytes, void* stream);
int64_t sgap_sddmm_csr_workspace_size(int64_t K, int64_t J, int window_kb, int max_long_rows);

/*
 * Tensor-times-matrix product along the last index of a third-order sparse
 * tensor, the TTM form of the paper's Section 2.1 (second form under Eq. 1):
 *   Y[i, j, l] = sum_k A[i, j, k] * X1[k, l].
 * A is stored as compressed sparse fibers in the index order (i, j, k); only
 * its fiber level enters the sum: fiber f (one stored (i, j) pair) owns the
 * entries eptr[f] .. eptr[f+1]-1 with third indices eidx[p] and values
 * vals[p].  The result is kept on A's stored fibers, one dense row per fiber:
 *   Yf[f, l] = sum_{p in fiber f} vals[p] * X1[eidx[p], l]
 * (rows of Y without a stored fiber are zero and are not materialised; the
 * caller's slice pointer and second-index arrays say which (i, j) a row
 * belongs to).  The reduction, along the sparse index k, is the one of SpMM
 * (Section 2.1), so every point of the SpMM design space applies.
 *   F         number of stored fibers
 *   K, L      extent of the contracted index, columns of X1 and Yf
 *   eptr      device, F+1 int32, eptr[0] = 0, non-decreasing
 *   eidx      device, eptr[F] int32 in [0, K)
 *   vals      device, eptr[F] floats
 *   X1        device, K x L row-major
 *   Yf        device, F x L row-major; OVERWRITTEN
 *   group_size, strategy, schedule, nnz_hint, stream, ownership, errors
 *             as for sgap_spmm_csr_ex with rows = fibers.
 */
int sgap_ttm_csf(int64_t F, int64_t K, int64_t L,
                 const int32_t* eptr, const int32_t* eidx, const float* vals,
                 const float* X1, float* Yf,
                 int group_size, int strategy, int schedule, int64_t nnz_hint, void* stream);

/*
 * Matricized tensor times Khatri-Rao product, the MTTKRP form of the paper's
 * Section 2.1 (first form under Eq. 1):
 *   Y[i, j] = sum_{k, l} A[i, k, l] * X1[k, j] * X2[l, j].
 * A (I x K x L) is stored as compressed sparse fibers in the index order
 * (i, k, l): slice i owns the fibers fptr[i] .. fptr[i+1]-1; fiber f has
 * second index fidx[f] and owns the entries eptr[f] .. eptr[f+1]-1; entry p
 * has third index eidx[p] and value vals[p].  The operator holds two
 * reductions of the SpMM kind, the first over the entries of a fiber, the
 * second over the fibers of a slice, whose input is the first one's output
 * (Section 2.1); both are served by the segment-group primitives.
 *   fptr      device, I+1 int32, fptr[0] = 0, non-decreasing
 *   fidx      device, fptr[I] int32 in [0, K)
 *   eptr      device, fptr[I]+1 int32, eptr[0] = 0, non-decreasing
 *   eidx      device, eptr[fptr[I]] int32 in [0, L)
 *   vals      device, as many floats
 *   X1, X2    device, K x J and L x J row-major
 *   Y         device, I x J row-major; OVERWRITTEN
 *   group_size, strategy
 *             SGAP_REDUCE_PARALLEL: group_size lanes share a slice, split its
 *             fibers between them and tree-sum once per slice;
 *             SGAP_REDUCE_SERIAL: one lane (per column chunk) works through
 *             group_size consecutive slices by itself.
 * Slices are the unit of work (row-split schedule): every element of Y has
 * one writer, no atomics, empty slices are written as zeros, results are
 * reproducible run to run.  Indices need not be sorted or distinct.
 * Asynchronous on `stream`; ownership and errors as for sgap_spmm_csr.
 * I == 0 or J == 0 returns at once.  fidx, eptr, eidx and vals may be null
 * only for a tensor without fibers (every fptr[i] = 0): they are read only
 * for fibers that fptr announces, which the host cannot check.
 */
int sgap_mttkrp_csf(int64_t I, int64_t K, int64_t L, int64_t J,
                    const int32_t* fptr, const int32_t* fidx,
                    const int32_t* eptr, const int32_t* eidx, const float* vals,
                    const float* X1, const float* X2, float* Y,
                    int group_size, int strategy, void* stream);

/*
 * The same operator with a choice of schedule (Section 6's two schedules
 * carried over to it):
 *   SGAP_SCHED_ROW_SPLIT     slices are the unit of work: exactly
 *                            sgap_mttkrp_csf (nnz_hint is not used)
 *   SGAP_SCHED_NNZ_BALANCED  stored entries are the unit of work, in tiles of
 *                            1,024, whatever slices and fibers they fall in (a
 *                            tensor with a few huge slices keeps the chip
 *                            busy).  parallel: G lanes hold G consecutive
 *                            entries and run two segmented sums, keyed by
 *                            fiber and then, over the fiber sums times their
 *                            rows of X1, by slice.  serial: a lane walks G
 *                            consecutive entries and closes fibers into the
 *                            slice's sum and slices into Y where they end.
 *                            Y is set to zero first and every run's sum is
 *                            added with fp32 atomics: results agree from run
 *                            to run within rounding only.
 *   nnz_hint   the number of stored entries if the host knows it (sizes the
 *              grid for small tensors), else -1
 * Everything else, and the errors, as sgap_mttkrp_csf; an unknown schedule is
 * SGAP_ERR_INVALID_ARG.
 */
int sgap_mttkrp_csf_ex(int64_t I, int64_t K, int64_t L, int64_t J, const int32_t* fptr, const int32_t* fidx,
                       const int32_t* eptr, const int32_t* eidx, const float* vals, const float* X1, const float* X2,
                       float* Y, int group_size, int strategy, int schedule, int64_t nnz_hint, void* stream);

/*
 * Tuner over the design space: the paper closes (Section 8) by proposing that
 * the space be exposed as an auto-tuning interface, and Table 5 measures what
 * a per-matrix choice gains over the best fixed point.  Times every
 * (group_size, strategy, schedule) point, 7 x 2 x 2 = SGAP_NUM_POINTS of them,
 * on the caller's operands with HIP events on `stream`, and reports the
 * fastest.  Each point runs once, timed, as a warm-up and,
 * unless that run was more than 4 times slower than the best point so far,
 * `reps` more times (reps >= 1); its time is the minimum over its timed runs and
 * includes the row-zeroing pass of the nnz-balanced schedule.
 *   table  host, NULL or room for SGAP_NUM_POINTS entries, filled in the order
 *          schedule (row-split first), strategy (parallel first), group size
 *          ascending.
 *   best   host, not NULL: the fastest point.
 * The tuning defaults in force (sgap_set_tuning) apply to the timed launches.
 * The call blocks until the measurements are done (it synchronises `stream`),
 * allocates no device memory and leaves in C the result of the fastest point,
 * computed last.  M == 0 or N == 0: nothing to time, SGAP_ERR_INVALID_ARG.
 * Other arguments and errors as for sgap_spmm_csr_ex.
 */
#define SGAP_NUM_POINTS 28
typedef struct {
    int group_size;
    int strategy;
    int schedule;
    float ms;
} sgap_point_time;
int sgap_autotune_csr(int64_t M, int64_t K, int64_t N,
                      const int32_t* rowptr, const int32_t* colidx, const float* vals,
                      const float* B, float* C, int64_t nnz_hint, int reps,
                      sgap_point_time* table, sgap_point_time* best, void* stream);

/*
 * The tuner over the whole space the library has (Section 7.2 tunes
 * <groupSz, blockSz, tileSz, workerDimR> per matrix, Tables 4 and 5).  Rates,
 * in this order: the SGAP_NUM_POINTS points above; the 21 row-split points
 * with the reduction narrower than the tiling (group_size 2..64, reduce_size
 * below it: Table 1); if `workspace` covers the default window and list
 * (sgap_spmm_csr_workspace_size with long_row_min > 0, window_kb = 0,
 * max_long_rows = 0), the row-split points with group sizes 1 to 8 of both
 * strategies with the long rows by column windows (long_row_min 512 and
 * 2048); then, around the fastest configuration so far, one knob at a time:
 * block_size 128 and 512, tile_cols 32, 64, 256, rows_per_group 1 to 16
 * (row-split parallel), wave_rows on and off (row-split serial), window_kb
 * 2048 and 4096 (window path, where the workspace covers it), or nnz_tile 512,
 * 1024, 2048 (nnz-balanced serial).
 * Timing of one configuration as in sgap_autotune_csr.
 *   workspace, workspace_bytes  as for sgap_spmm_csr_cfg; NULL/0: the window
 *          path is not rated
 *   table  host, NULL or room for `capacity` entries; the first `capacity`
 *          rated configurations in the order above
 *   count  host or NULL: how many configurations were rated (may exceed
 *          capacity; at most SGAP_MAX_TUNED_POINTS)
 *   best   host, not NULL: the fastest configuration and its time; it can be
 *          handed to sgap_spmm_csr_cfg as it is
 * Blocks, allocates nothing and leaves the fastest configuration's result in C.
 */
#define SGAP_MAX_TUNED_POINTS 96
typedef struct {
    sgap_config config;
    float ms;
} sgap_tuned_point;
int sgap_autotune_csr_cfg(int64_t M, int64_t K, int64_t N,
                          const int32_t* rowptr, const int32_t* colidx, const float* vals,
                          const float* B, float* C, int64_t nnz_hint, int reps,
                          void* workspace, int64_t workspace_bytes,
                          sgap_tuned_point* table, int capacity, int* count,
                          sgap_tuned_point* best, void* stream);

/* Text for a status code / detail of this thread's last failure (static or
 * thread-local storage; never free). */
const char* sgap_status_string(int status);
const char* sgap_last_error(void);

/* Library version: major*10000 + minor*100 + patch. */
int sgap_version(void);

/*
 * Process-wide defaults for the tiling choices of the entry points that take
 * no sgap_config (sgap_spmm_csr, _ex, _gr, sgap_ttm_csf, sgap_autotune_csr),
 * in the spirit of the paper's Section 7.2 (tiling parameters are separate
 * from the synchronisation granularity).  Not thread-safe; value 0 (or -1
 * where stated) restores the automatic choice.  They change speed only, never
 * results beyond fp32 summation order.  sgap_spmm_csr_cfg ignores them.
 *   SGAP_TUNE_TILE_COLS  columns of B/C per work item of the row-split
 *                        schedule (rounded up to the vector width, capped at
 *                        N); 0 = automatic.
 *   SGAP_TUNE_XCD_REMAP  1/-1: hand each of the 8 dies a contiguous run of
 *                        work items so that its L2 keeps the rows of B it
 *                        gathers; 0: plain round-robin order.
 *   SGAP_TUNE_ROWS_PER_GROUP  rows one group works through per
 *                        work item in the row-split parallel strategy (the
 *                        serial strategy takes group_size rows by definition);
 *                        0 = automatic, from the mean row length.  Also the
 *                        slices per group of sgap_mttkrp_csf's parallel strategy
 *                        (automatic: about 16 slices per workgroup).
 *   SGAP_TUNE_PERSISTENT 1: the row-split schedule launches only as many
 *                        workgroups as the chip holds at once and each loops
 *                        over work items; 0 (default): one workgroup per item.
 *   SGAP_TUNE_NNZ_TILE   stored entries per tile of the nnz-balanced serial
 *                        strategy: 256, 512, 1024 or 2048 (the two small ones
 *                        need N % 4 == 0 and 16-byte aligned B and C, else
 *                        the automatic choice is kept); 0 = automatic, from
 *                        nnz and the size of the chip.
 *   SGAP_TUNE_SDDMM_ROW_CACHE  1 (default): sgap_sddmm_csr's parallel strategy
 *                        hands a group consecutive stored entries and keeps
 *                        the current row of X1 in registers when
 *                        J <= 16 * group_size and the operands are 16-byte
 *                        aligned; 0: every entry loads both of its rows.
 * Knobs 6 and 7 (long rows by column windows) of earlier versions are gone:
 * that path needs working memory and is chosen per call, see sgap_config;
 * their numbers are refused with SGAP_ERR_INVALID_ARG.
 */
typedef enum {
    SGAP_TUNE_TILE_COLS = 0,
    SGAP_TUNE_XCD_REMAP = 1,
    SGAP_TUNE_ROWS_PER_GROUP = 2,
    SGAP_TUNE_PERSISTENT = 3,
    SGAP_TUNE_NNZ_TILE = 4,
    SGAP_TUNE_SDDMM_ROW_CACHE = 5
} sgap_tuning_knob;
int sgap_set_tuning(int knob, int value);

/*
 * Check the preconditions that the compute calls rely on and cannot test
 * themselves (the paper's Section 2.2 takes a well-formed CSR for granted).
 * Debugging aid: it runs three small kernels and then WAITS for `stream`.
 *   nnz       the length of colidx (required here: a damaged rowptr must not
 *             decide how far colidx is read)
 *   report    host, 4 counters:
 *             [0] defects of rowptr: rowptr[0] != 0, rowptr[M] != nnz, and
 *                 every i with rowptr[i] > rowptr[i+1]
 *             [1] stored entries whose column is outside [0, K)
 *             [2] stored entries that are not larger than their predecessor
 *                 in the same row (unsorted or repeated columns: allowed, all
 *                 kernels just add; counted only when [0] is zero, else -1)
 *             [3] rows without stored entries (information; -1 unless [0] is zero)
 * Returns SGAP_OK when the check ran (whatever it found), SGAP_ERR_INVALID_ARG
 * for null pointers with non-zero extents or negative sizes.  The counters
 * live in a small device array of the library: calls must not overlap on one
 * GPU.
 */
int sgap_validate_csr(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colidx, int64_t nnz,
                      int64_t* report, void* stream);

/*
 * Row order (optional preprocessing; the schedules of Section 6 take the rows
 * in the order in which they are stored, and Section 2.2 names the work on
 * locality and balance that a better order stands for).  Writes a copy of the
 * CSR matrix whose rows are grouped by a coarse key, smaller key first, rows of
 * equal key in no particular order:
 *   SGAP_ORDER_BY_FIRST_COLUMN  key = floor(first stored column * 4096 / K);
 *                               rows without stored entries last (key 4096)
 *   SGAP_ORDER_BY_LENGTH        key = 4096 - min(stored entries, 4096): the
 *                               longest rows first, rows without entries last
 * The stored entries of a row keep their order.  The product of the new
 * matrix comes out in the new row order: row j of A' * B is row perm[j] of
 * A * B.
 *   rowptr, colidx, vals   device, the matrix as for sgap_spmm_csr; read only
 *   perm                   device, M: perm[j] = the row of A that is row j of A'
 *   rowptr_out             device, M+1
 *   colidx_out, vals_out   device, nnz = rowptr[M] each; must not overlap the inputs
 *                          (these two and colidx, vals may be null only when
 *                          the matrix has no stored entries: the host cannot check)
 *   workspace              device, at least sgap_reorder_rows_workspace_size(M)
 *                          bytes, 16-byte aligned, caller-owned, contents
 *                          meaningless before and after; calls that overlap in
 *                          time need a workspace each
 * Asynchronous on `stream`; allocates nothing.  M == 0 writes rowptr_out[0] = 0.
 * Errors: SGAP_ERR_INVALID_ARG (negative sizes, M beyond the int32 row range,
 * K < 1 with M > 0, unknown order, null rowptr, rowptr_out or perm, workspace
 * too small or misaligned) launches nothing; SGAP_ERR_HIP as for the compute calls.
 * sgap_reorder_rows_workspace_size returns -1 for a negative M.
 */
typedef enum { SGAP_ORDER_BY_FIRST_COLUMN = 0, SGAP_ORDER_BY_LENGTH = 1 } sgap_row_order;
int64_t sgap_reorder_rows_workspace_size(int64_t M);
int sgap_reorder_rows_csr(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colidx, const float* vals,
                          int order, int32_t* perm, int32_t* rowptr_out, int32_t* colidx_out, float* vals_out,
                          void* workspace, int64_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SGAP_H */
