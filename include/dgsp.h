/*
 * libdgsp - CSR sparse x dense multiplication for AMD MI355X (gfx950), fp32.
 *
 * C-ABI of the hot path of "Efficient Sparse Matrix Kernels based on Adaptive
 * Workload-Balancing and Parallel-Reduction" (arXiv 2106.16064):
 *
 *     Y[M x N] = A[M x K] * X[K x N]        (Section 1; N = 1 is SpMV)
 *
 * with A in CSR and X, Y dense.  Four kernels span the paper's design space
 * (Section 2.1): {row-split, nnz-balanced} x {sequential, parallel reduction};
 * a rule-based selector (Section 2.2) picks one from N and two row-length
 * statistics.
 *
 * Conventions for every entry point
 *   - "device" pointers are HIP device memory of the current device, "host"
 *     pointers ordinary host memory.  The caller owns every buffer; the
 *     library allocates nothing on the device and keeps no state between
 *     calls apart from the selector thresholds (dgsp_set_thresholds) and the
 *     64-byte static device array of dgsp_features_from_csr_device_noalloc.
 *   - Indices are int32, zero based.  Values are fp32, accumulation is fp32
 *     (the paper's float2/float4 loads, Section 2.1.2, imply single
 *     precision).  The summation order differs between kernels, so results
 *     agree with an exact sum to within c*eps32*(|A||X|) elementwise, not bit
 *     for bit; the nnz-balanced kernels combine partial rows with fp32 atomic
 *     adds and are not run-to-run bit-reproducible.
 *   - X and Y are row-major (the layout Section 2.1.2 needs: X[k,0], X[k,1]
 *     adjacent) with leading dimension N unless an entry point takes ldx, ldy.
 *   - Calls are asynchronous unless stated otherwise: work is enqueued on
 *     `stream` (a hipStream_t passed as void*, NULL = the default stream) and
 *     the call returns.  dgsp_features_from_csr_device and dgsp_autotune wait
 *     for their work because they hand results back in host memory.
 *   - Return value: a dgsp_status_t.  On any error nothing has been enqueued.
 */
#ifndef DGSP_H
#define DGSP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The four design points of Section 2.1 (Figure 1 of the paper). */
typedef enum {
    DGSP_RS_SR = 0, /* row-split, sequential reduction; sparse rows staged in LDS
                       (coalesced sparse-row caching, Section 2.1.3)            */
    DGSP_RS_PR = 1, /* row-split, parallel reduction (CSR-Vector lineage) with
                       vector-type dense-row loads (Section 2.1.2)              */
    DGSP_NB_SR = 2, /* nnz-balanced, sequential reduction, LDS-staged tiles      */
    DGSP_NB_PR = 3, /* nnz-balanced, parallel reduction: wave64 vectorized
                       segment reduction (Section 2.1.1)                        */
    DGSP_AUTO = -1  /* let the library choose (see each entry point)            */
} dgsp_algo_t;

typedef enum {
    DGSP_OK = 0,
    DGSP_ERR_INVALID_ARG = 1, /* negative extent, NULL pointer with non-zero extent,
                                 unknown algo, extent beyond the int32 index range   */
    DGSP_ERR_UNSUPPORTED = 2, /* valid arguments outside a stated limit of the kernel asked
                                 for (ldy beyond 2^20 in the balanced kernels; a measurement
                                 switch the kernel does not offer)                   */
    DGSP_ERR_LAUNCH = 3       /* the HIP runtime refused a launch                    */
} dgsp_status_t;

/* Row-length statistics of a CSR matrix, the selector's input (Section 2.2:
 * avg_row and stdv_row; cv_row = stdv_row / avg_row is the paper's combined
 * metric).  stdv_row is the population standard deviation over all M rows,
 * empty rows included. */
typedef struct {
    int64_t M, K, nnz;
    double avg_row, stdv_row, cv_row;
    int64_t max_row, min_row;
    double col_span; /* mean over non-empty rows of (largest - smallest column + 1) / K; 0 = unknown.
                        Not part of the paper's rules.  It tells the sequential kernels how many
                        dense-row loads to keep in flight (a banded matrix, col_span <= 0.05, re-uses
                        rows of X between neighbouring rows and wants more), and the added
                        large-dense-operand rule of the selector looks at it (see below). */
} dgsp_features_t;

/* Selector thresholds (Section 2.2 says they are set empirically and prints no
 * values; the defaults were fitted on MI355X).
 *   N <= n_parallel_max          -> parallel reduction, else sequential
 *   parallel:  avg_row >= pr_avg_row_min AND cv_row <= pr_cv_max AND
 *              nnz < pr_nnz_max -> row-split, else nnz-balanced (the last two
 *              conditions are additions: the paper's parallel-side rule looks at
 *              avg_row only.  The balanced kernel streams faster but needs a
 *              second, small launch, which pays off from some ten million stored
 *              entries on.  Set pr_cv_max to a huge value and
 *              pr_nnz_max to INT64_MAX to get the paper's rule verbatim)
 *   sequential: cv_row > sr_cv_min AND stdv_row > sr_stdv_min -> nnz-balanced,
 *              else row-split (the paper's metric is cv_row alone; the second
 *              condition is an addition: with short rows even a large cv_row
 *              leaves no row long enough to stall a wave; set sr_stdv_min to 0
 *              for the paper's rule verbatim)
 *   up to eight columns (an addition): n_parallel_max < N <= wide_parallel_n
 *              AND the sequential side would balance -> nnz-balanced PARALLEL
 *              kernel.  That kernel reads eight dense columns per lane with two
 *              dwordx4 accesses (for N = 5, 6, 7 the two overlap), so these N are
 *              still one pass over the sparse matrix, and it beat the balanced
 *              sequential kernel by 6-31 % there.  Meant for 8; 0 switches it off.
 *   short rows (an addition, checked first, at every N): avg_row <=
 *              short_avg_row_max AND max_row <= short_max_row_max -> row-split
 *              sequential.  When no row is long, one lane group per row keeps the
 *              whole wave busy for max_row steps with no cross-lane step and no
 *              long-row tail; it beat the other three kernels on every such
 *              matrix measured with enough rows.  It applies only when the rows fill the
 *              machine: the row-split sequential kernel runs M * (lanes per row at this N)
 *              / 64 waves, and with fewer than short_min_waves of them (65 536 rows at
 *              N <= 4 are 1024 waves) most CUs hold a single wave; such matrices go on to
 *              the rules below.  Set short_avg_row_max to 0 to switch the rule off,
 *              short_min_waves to 0 to apply it at any size.
 *   small matrix, parallel side (an addition): N <= n_parallel_max AND nnz <=
 *              pr_small_nnz_max AND cv_row <= pr_small_cv_max -> row-split parallel.  The
 *              balanced kernels need a second, small launch (4-6 us); for a matrix whose
 *              whole multiplication takes 12-20 us the single launch wins when no row is
 *              much longer than the others (27-point stencil on 40^3: 12-14 against
 *              19-20 us).  pr_small_nnz_max 0 switches it off.
 *   large dense operand (an addition, checked second, on the parallel side
 *              N <= n_parallel_max only): K * N * 4 >= big_x_bytes_min AND
 *              cv_row <= big_x_cv_max AND avg_row <= big_x_avg_row_max AND
 *              col_span >= 0.5 -> row-split sequential.  When X no longer fits
 *              one XCD's 4 MB L2, rows of about equal length whose ascending
 *              columns spread over most of K are swept in step by the lanes of
 *              a wave, one row per lane, so the part of X in use at a time stays
 *              small; the parallel kernels spread one row over the lanes and touch
 *              all of X at once (measured 10-80 % slower there).  Needs col_span;
 *              big_x_bytes_min 0 switches it off.  */
typedef struct {
    int64_t n_parallel_max;
    double pr_avg_row_min;
    double pr_cv_max;
    double sr_cv_min;
    double sr_stdv_min;
    int64_t pr_nnz_max;
    double short_avg_row_max;
    int64_t short_max_row_max;
    int64_t wide_parallel_n;
    int64_t big_x_bytes_min;
    double big_x_cv_max;
    double big_x_avg_row_max;
    int64_t short_min_waves;
    int64_t pr_small_nnz_max;
    double pr_small_cv_max;
} dgsp_thresholds_t;

/*
 * Y = A X (Section 1), one of the four kernels of Section 2.1.
 *
 *   M, K, N   extents, all >= 0; M + 1 and nnz must fit int32.
 *   rowptr    device, int32[M+1], rowptr[0] = 0, non-decreasing, rowptr[M] = nnz.
 *   colidx    device, int32[nnz], 0 <= colidx[p] < K; any order inside a row,
 *             repeated (row, col) pairs add.  Out-of-range indices are
 *             undefined behaviour (not checked on the device).
 *   vals      device, fp32[nnz].
 *   X         device, fp32[K*N], row-major, ld = N.  Read only.
 *   Y         device, fp32[M*N], row-major, ld = N.  Overwritten (alpha = 1,
 *             beta = 0); rows of A without entries give exact zeros.  Must not
 *             overlap X.
 *   algo      a dgsp_algo_t.  DGSP_AUTO here, where no features are known,
 *             means: nnz-balanced, parallel reduction if N <= max(n_parallel_max,
 *             wide_parallel_n) (8 by default: one pass over the matrix), else
 *             nnz-balanced sequential (the variants that are safe for any
 *             row-length distribution).
 *   stream    hipStream_t as void*, NULL = default stream.
 *
 * Every algo accepts every N >= 1 and any (float) alignment of X and Y; no
 * vector path depends on alignment or on the leading dimensions.  The
 * parallel-reduction kernels load v dense values per entry, v the widest of
 * 4, 3, 2, 1 that divides N (8 as two accesses in DGSP_NB_PR when 8 divides
 * N), and make one pass over A per v columns; the sequential-reduction kernels
 * give a lane four columns for every N >= 4 except 6.  What the layout still
 * decides is how many 128-byte lines a row of X spans: rows that start on
 * line boundaries (ldx a multiple of 32) are fetched with the fewest requests
 * (N = 31 with ldx = 32 ran 1.2-1.5x faster than with ldx = 31).
 * M == 0 or N == 0: returns DGSP_OK without launching.  The number of stored
 * entries is read on the device from rowptr[M]; the call never synchronises.
 */
int dgsp_spmm_csr(int64_t M, int64_t K, int64_t N,
                  const int32_t *rowptr, const int32_t *colidx, const float *vals,
                  const float *X, float *Y, int algo, void *stream);

/*
 * Same operation with the number of stored entries supplied by the caller
 * (nnz >= 0 must equal rowptr[M]; nnz < 0 means unknown and makes this call
 * identical to dgsp_spmm_csr).  Knowing nnz lets the host size the launch to
 * the work (small matrices get small grids) and pick the lanes-per-row of the
 * row-split parallel kernel from nnz / M before the launch instead of inside
 * the kernel.  The result is the same.
 */
int dgsp_spmm_csr_nnz(int64_t M, int64_t K, int64_t N, int64_t nnz,
                      const int32_t *rowptr, const int32_t *colidx, const float *vals,
                      const float *X, float *Y, int algo, void *stream);

/*
 * Adaptive call (Section 2.2): dgsp_select_algo(features, N), then the chosen
 * kernel.  `features` is a host pointer, read before the call returns.  If
 * `chosen` is not NULL it receives the dgsp_algo_t that ran.
 */
int dgsp_spmm_csr_auto(int64_t M, int64_t K, int64_t N,
                       const dgsp_features_t *features,
                       const int32_t *rowptr, const int32_t *colidx, const float *vals,
                       const float *X, float *Y, int *chosen, void *stream);

/*
 * Kernel-selection rules of Section 2.2 (the decision-tree figure): first N decides parallel vs sequential reduction, then avg_row
 * (parallel side) or stdv_row / avg_row (sequential side) decides whether to
 * balance by non-zeros.  Pure host function; returns a dgsp_algo_t in 0..3, or
 * DGSP_AUTO (-1) if features is NULL or N < 1.
 */
int dgsp_select_algo(const dgsp_features_t *features, int64_t N);

/* Read / replace the thresholds used by dgsp_select_algo (process-wide; reads
 * and writes are serialised by a lock, every selection sees one consistent set).
 * They steer the CHOICE of kernel only: the launch geometry of a kernel asked for
 * by name does not depend on them.  Host pointers. */
void dgsp_get_thresholds(dgsp_thresholds_t *out);
void dgsp_set_thresholds(const dgsp_thresholds_t *in);

/*
 * Row-length statistics from a HOST copy of rowptr (the cheap features of
 * Section 2.2: one pass over M+1 integers, two accumulators).  Returns
 * DGSP_ERR_INVALID_ARG if M < 0, a pointer is NULL, rowptr[0] != 0 or rowptr
 * decreases.  M == 0 gives all-zero features.
 */
int dgsp_features_from_rowptr_host(int64_t M, int64_t K, const int32_t *rowptr_host,
                                   dgsp_features_t *out);

/*
 * Same statistics plus col_span, from HOST copies of rowptr and colidx (one more
 * pass, over the two ends of every sorted row; unsorted rows are scanned).
 */
int dgsp_features_from_csr_host(int64_t M, int64_t K, const int32_t *rowptr_host,
                                const int32_t *colidx_host, dgsp_features_t *out);

/*
 * The same statistics from a matrix that lives in DEVICE memory: one pass over
 * rowptr (and, if colidx is not NULL, over every row's columns for col_span; a
 * NULL colidx leaves col_span 0).  All sums are integer sums, so the result equals
 * dgsp_features_from_csr_host on a host copy bit for bit.
 *   rowptr, colidx  device, as in dgsp_spmm_csr
 *   workspace       device, DGSP_FEATURES_WORKSPACE_BYTES bytes, 8-byte aligned,
 *                   caller-owned, overwritten; needs no initialisation
 *   out             host
 * The call enqueues two small launches and a copy on `stream` and WAITS for them
 * (the result goes to host memory).  Errors as the host versions; a NULL or
 * misaligned workspace with M > 0 -> DGSP_ERR_INVALID_ARG.
 */
#define DGSP_FEATURES_WORKSPACE_BYTES 64
int dgsp_features_from_csr_device(int64_t M, int64_t K, const int32_t *rowptr, const int32_t *colidx,
                                  void *workspace, dgsp_features_t *out, void *stream);

/*
 * For callers that cannot allocate device memory or pass a workspace (code under
 * HIP graph capture set-up, tight serving loops, harnesses that forbid hipMalloc):
 * the same statistics as dgsp_features_from_csr_device with the 64 bytes of
 * scratch in a static device array inside the library instead of a caller
 * workspace.  No hipMalloc / hipFree or other allocating call is made.
 *   - Limit: M <= DGSP_FEATURES_NOALLOC_MAX_ROWS (the int32 index range the
 *     library has anyway; the scratch itself is 64 bytes whatever M is); larger M,
 *     negative extents or NULL pointers -> DGSP_ERR_INVALID_ARG, nothing enqueued.
 *   - Every call on one GPU uses that GPU's one array, cleared by a small kernel at
 *     the start of each call: calls that overlap on one GPU (different streams or
 *     threads) race and give wrong statistics.  Calls on different GPUs do not
 *     interfere (each device holds its own copy, found once per device on first use).
 *   - Like the workspace version it WAITS for its launches (result in host memory).
 */
#define DGSP_FEATURES_NOALLOC_MAX_ROWS (2147483647LL - 4096LL)
int dgsp_features_from_csr_device_noalloc(int64_t M, int64_t K, const int32_t *rowptr, const int32_t *colidx,
                                          dgsp_features_t *out, void *stream);

/*
 * Profile-based selection (Section 3.1 names running all kernels once off-line
 * and keeping the fastest as the alternative to the rules): runs each of the four
 * kernels on the given buffers - one untimed call, then `reps` (clamped to
 * 1..100) calls bracketed by events on `stream` - and reports the fastest.
 *   ms    host, 4 floats or NULL: best time of each kernel in milliseconds,
 *         indexed by dgsp_algo_t (INFINITY for a kernel that rejects the shape)
 *   best  host, receives the dgsp_algo_t with the smallest time
 * Other arguments as dgsp_spmm_csr_phase.  Y is overwritten with the product
 * (every kernel computes the same one).  The call WAITS for its launches; it
 * allocates no device memory.  Errors of the kernels are passed on.
 */
int dgsp_autotune(int64_t M, int64_t K, int64_t N, int64_t nnz,
                  const int32_t *rowptr, const int32_t *colidx, const float *vals,
                  const float *X, float *Y, const dgsp_features_t *features,
                  int reps, float *ms, int *best, void *stream);

/*
 * The same multiplication for matrices whose row pointers are 64-bit (the paper leaves the index type open;
 * this is for more than 2^31 - 4096 stored entries, which the other entry points reject).  Column indices stay
 * int32 (K within the int32 range), as do M and N.
 *   rowptr     device, int64[M+1], rowptr[0] = 0, non-decreasing, rowptr[M] = nnz
 *   nnz        the number of stored entries (>= 0; it sizes the workspace, so the caller has to know it)
 *   workspace  device, dgsp_spmm_csr_i64_workspace_bytes(M, nnz) bytes (4 (M + 1) and a few hundred more),
 *              16-byte aligned, caller-owned, overwritten
 * How: the rows are cut into slabs that hold about 2^30 entries each; per slab a small launch writes 32-bit row
 * pointers relative to the slab's first entry into the workspace, and the chosen kernel runs on the slab (its
 * rows of Y are disjoint from every other slab's).  No row may hold 2^30 entries or more, and at most 15 slabs
 * are taken: else DGSP_ERR_UNSUPPORTED.  The slab cuts are found on the device and decide launch sizes, so the
 * call WAITS once for `stream` (a 200-byte copy) before it enqueues the slabs; it returns after enqueueing them.
 * algo: one of the four kernels, or DGSP_AUTO = the balanced kernel for the width, as in dgsp_spmm_csr.
 * Other arguments, result and errors as dgsp_spmm_csr_nnz; a wrong nnz or rowptr[0] != 0 -> DGSP_ERR_INVALID_ARG.
 */
int dgsp_spmm_csr_i64(int64_t M, int64_t K, int64_t N, int64_t nnz,
                      const int64_t *rowptr, const int32_t *colidx, const float *vals,
                      const float *X, float *Y, int algo,
                      void *workspace, int64_t workspace_bytes, void *stream);
int64_t dgsp_spmm_csr_i64_workspace_bytes(int64_t M, int64_t nnz);

/*
 * Measurement aid: the same multiplication, one step at a time.  The two
 * nnz-balanced kernels are two launches per call - a small "prepare" launch
 * (zeroes the rows that are later combined with atomic adds) and the main
 * kernel.  A profiler sees them apart; a benchmark that brackets launches with
 * events needs this entry to time the main kernel alone.
 *   phase = DGSP_PHASE_ALL      same as dgsp_spmm_csr_nnz
 *           DGSP_PHASE_PREPARE  only the prepare launch (no-op for row-split algos)
 *           DGSP_PHASE_MAIN     only the main kernel; the result is right only if
 *                               PREPARE for the same arguments ran before it on
 *                               the same stream
 * algo must be one of the four kernels (not DGSP_AUTO).  `features` may be NULL;
 * if given (host pointer) its nnz and col_span are used as in the adaptive call.
 */
typedef enum { DGSP_PHASE_ALL = 0, DGSP_PHASE_PREPARE = 1, DGSP_PHASE_MAIN = 2 } dgsp_phase_t;
int dgsp_spmm_csr_phase(int64_t M, int64_t K, int64_t N, int64_t nnz,
                        const int32_t *rowptr, const int32_t *colidx, const float *vals,
                        const float *X, float *Y, int algo, int phase,
                        const dgsp_features_t *features, void *stream);

/*
 * The same multiplication on strided views: row k of X starts at X + k*ldx, row i
 * of Y at Y + i*ldy (in floats; ldx >= N and ldy >= N, else DGSP_ERR_INVALID_ARG).
 * Only the N used columns of a row are read or written; what lies between rows is
 * not touched.  This is what a column slice of a wider row-major matrix needs
 * (the dense columns shared out between devices, or processed a slice at a time).
 * The vector width of the dense-row accesses (Section 2.1.2) depends on N only,
 * not on ldx, ldy or the alignment of the views (see dgsp_spmm_csr); rows that
 * start on 128-byte lines are merely fetched with fewer requests.  algo may be
 * DGSP_AUTO: with features the rules choose, without them the balanced kernel
 * for the width; where ldy exceeds the balanced kernels' limit of 2^20 floats the
 * library's own choice falls to DGSP_RS_SR (a balanced kernel asked for by name
 * returns DGSP_ERR_UNSUPPORTED there).  Everything else as dgsp_spmm_csr_nnz;
 * `features` may be NULL (host pointer otherwise).
 */
int dgsp_spmm_csr_ld(int64_t M, int64_t K, int64_t N, int64_t nnz,
                     const int32_t *rowptr, const int32_t *colidx, const float *vals,
                     const float *X, int64_t ldx, float *Y, int64_t ldy, int algo,
                     const dgsp_features_t *features, void *stream);

/*
 * The scaled form  Y = alpha * (A X) + beta * Y  on strided views (the paper
 * computes Y = A X; this is the usual BLAS-style generalisation, computed by
 * variants of the same four kernels that scale a row's sum as they write it).
 * With beta == 0 the old contents of Y are not read (they may be anything,
 * NaN included).  Rows of A without entries give beta * Y.  Rows whose partial
 * sums meet through atomic adds are first multiplied by beta by the prepare
 * launch.  Other
 * arguments, vector-width rule and algo == DGSP_AUTO as in dgsp_spmm_csr_ld.
 */
int dgsp_spmm_csr_axpby(int64_t M, int64_t K, int64_t N, int64_t nnz,
                        const int32_t *rowptr, const int32_t *colidx, const float *vals,
                        const float *X, int64_t ldx, float *Y, int64_t ldy,
                        float alpha, float beta, int algo,
                        const dgsp_features_t *features, void *stream);

/*
 * Measurement aid: the same multiplication with one of the paper's optimisations
 * switched off, for the comparisons of Sections 2.1.2 and 2.1.3.  Same arguments,
 * layouts, result and error behaviour as dgsp_spmm_csr_nnz; `switches` is a
 * bit-wise OR of
 *   DGSP_ABL_SCALAR_DENSE_LOADS  dense rows are read one float at a time, so a
 *                                parallel-reduction SpMM becomes N passes over the
 *                                sparse matrix, one per dense column: the
 *                                "N times SpMV" that vector-type dense-row loading
 *                                is measured against (Section 2.1.2).  Any algo.
 *   DGSP_ABL_NO_SPARSE_STAGING   sequential reduction without the LDS tile: every
 *                                lane reads colidx/vals from memory itself, the
 *                                "pure sequential reduction" that coalesced
 *                                sparse-row caching is measured against
 *                                (Section 2.1.3).  Only DGSP_RS_SR, else
 *                                DGSP_ERR_UNSUPPORTED.
 *   DGSP_ABL_ITEM_TILES          the balanced parallel kernel with its chunks cut into tiles of
 *                                merge-path items (entries + row ends), where a tile's gathers can
 *                                only be requested after the previous tile's row ends are counted.
 *   DGSP_ABL_ENTRY_BLOCKS        the balanced parallel kernel walking blocks of entries instead, whose
 *                                addresses are known ahead, with the next block's gathers in flight during
 *                                the row logic.  DGSP_NB_PR itself takes entry blocks at up to four dense
 *                                columns per lane from six million entries on unless the features say the matrix
 *                                is banded (col_span <= 0.05), and item tiles otherwise;
 *                                the two switches force one or the other: the comparison for that choice.
 *                                Only DGSP_NB_PR (entry blocks: only at widths that run up to four columns
 *                                per lane, i.e. not where N is a multiple of 8 or N = 5, 6, 7), not both, else
 *                                DGSP_ERR_UNSUPPORTED.
 *   DGSP_ABL_SERIAL_SEGMENT_SCAN the balanced parallel kernel with its segment reduction done as a serial
 *                                scan: the lanes' partial sums go to LDS and one lane adds them up in order,
 *                                starting afresh at every row boundary.  Same balanced split, same loads: the
 *                                workload-balanced design point WITHOUT the vectorized reduction, the third
 *                                alternative that Section 2.1.1 measures its segment reduction against
 *                                (beside row-split sequential and row-split parallel, which are DGSP_RS_SR and
 *                                DGSP_RS_PR).  Only DGSP_NB_PR at widths that run one or two dense columns per
 *                                lane (N = 1, 2, other N that 3 and 4 do not divide, or any N together with
 *                                DGSP_ABL_SCALAR_DENSE_LOADS), not with DGSP_ABL_ITEM_TILES; else
 *                                DGSP_ERR_UNSUPPORTED.  It runs on the entry-block pipeline at any size, so
 *                                it is to be held against DGSP_ABL_ENTRY_BLOCKS.
 *   DGSP_ABL_COLUMN_BLOCKS_32    the balanced sequential kernel with column blocks of 32 dense columns (one
 *                                128-byte line of a row of X per entry and block) instead of 64, where N is a
 *                                multiple of 32 from 64 on (ignored elsewhere): more passes over the sparse
 *                                matrix against a smaller slice of X per pass.
 *   DGSP_ABL_BLOCKS_OFF_XCDS     the balanced sequential kernel with its column blocks as a second grid
 *                                dimension, any XCD taking any block.  DGSP_NB_SR itself, when N >= 128 makes
 *                                2 or 4 column blocks, lets every XCD work on one block only, so that an L2
 *                                sees one block's slice of X (with 8 blocks that measured slower).  Both switches are comparisons for the layout
 *                                of the wide-N path (Section 2.1.3's kernel at N >= 64) and only go with
 *                                DGSP_NB_SR, else DGSP_ERR_UNSUPPORTED.
 * Unknown bits -> DGSP_ERR_INVALID_ARG.  algo must be one of the four kernels.
 * `features` may be NULL (host pointer otherwise; nnz and col_span are used).
 */
#define DGSP_ABL_SCALAR_DENSE_LOADS 1
#define DGSP_ABL_NO_SPARSE_STAGING 2
#define DGSP_ABL_ITEM_TILES 4
#define DGSP_ABL_SERIAL_SEGMENT_SCAN 8
#define DGSP_ABL_COLUMN_BLOCKS_32 16
#define DGSP_ABL_BLOCKS_OFF_XCDS 32
#define DGSP_ABL_ENTRY_BLOCKS 64
int dgsp_spmm_csr_ablation(int64_t M, int64_t K, int64_t N, int64_t nnz,
                           const int32_t *rowptr, const int32_t *colidx, const float *vals,
                           const float *X, float *Y, int algo, int switches,
                           const dgsp_features_t *features, void *stream);

/*
 * Measurement aid, not part of the method: out[t] = sum of x[idx[i]] over the
 * i that thread t visits (device buffers; idx int32[n] with 0 <= idx[i] < the
 * length of x; out fp32[dgsp_gather_probe_out_len()]).  It does nothing but
 * stream idx and gather from x, so its time is a floor for any kernel that
 * has to gather one dense value per stored entry (Section 2.1.2 names the
 * scattered dense-vector reads as the cost of parallel-reduction SpMV): run on
 * a matrix's colidx it gives the rate at which this machine can serve that
 * matrix's access pattern at all.
 */
int dgsp_gather_probe(float *out, const float *x, const int32_t *idx, int64_t n, void *stream);
int64_t dgsp_gather_probe_out_len(void);

/*
 * Measurement aids, not part of the method: the memory side of the kernels with no row logic at all, as floors
 * to hold the kernels against (Section 2.1.2 names the scattered dense reads as the cost of the parallel
 * reduction, Section 2.1.3 the contiguous dense-row reads as the strength of the sequential one).  All read
 * colidx (and vals) once, in order, and X where the columns say; none knows about rows.
 *   DGSP_PROBE_GATHER             N = 1: dgsp_gather_probe (stream colidx, gather x[colidx], nothing else)
 *   DGSP_PROBE_STREAM_GATHER_FMA  N in {1, 2, 4}: stream colidx and vals in blocks of 512 entries, gather N
 *                                 values of X per entry with one vector load, multiply-add; the load pipeline of
 *                                 the balanced parallel kernel (while a block is multiplied the next block's
 *                                 gathers and the entries of the block after are in flight)
 *   DGSP_PROBE_ROW_GATHER         N a multiple of 4: entries staged in LDS 512 at a time, lane groups walk them
 *                                 and load 16 bytes of the entry's row of X per lane (64 columns per group at most,
 *                                 further columns as further blocks): the walk of the sequential-reduction
 *                                 kernels without rows
 * colidx, vals: device, nnz entries, 0 <= colidx < K.  X: device, fp32 K x N row-major, ld = N.  out: device,
 * dgsp_floor_probe_out_len(mode, N) floats (-1: mode / N not offered), overwritten with the per-thread partial
 * sums: their total equals the sum over all entries p and columns n of vals[p] * X[colidx[p], n] (for
 * DGSP_PROBE_GATHER: of X[colidx[p]]), which is also the sum of all elements of A X.
 * Errors: DGSP_ERR_UNSUPPORTED for an N the mode does not offer, DGSP_ERR_INVALID_ARG otherwise.
 */
typedef enum { DGSP_PROBE_GATHER = 0, DGSP_PROBE_STREAM_GATHER_FMA = 1, DGSP_PROBE_ROW_GATHER = 2 } dgsp_probe_mode_t;
int dgsp_floor_probe(int mode, int64_t nnz, int64_t K, int64_t N, const int32_t *colidx, const float *vals,
                     const float *X, float *out, void *stream);
int64_t dgsp_floor_probe_out_len(int mode, int64_t N);

/*
 * Measurement aid, not part of the method: dst[i] = src[i] for i < n (device
 * fp32 buffers, n >= 0), a plain streaming copy whose 8*n bytes calibrate the
 * achievable HBM bandwidth and the profiler's byte counters.
 */
int dgsp_copy_f32(float *dst, const float *src, int64_t n, void *stream);

/* Static strings; never NULL. */
const char *dgsp_algo_name(int algo);
const char *dgsp_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* DGSP_H */
