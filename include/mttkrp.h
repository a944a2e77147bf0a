/*
 * mttkrp.h -- C ABI of the MI355X (gfx950) matrix-free dense MTTKRP library.
 *
 * The one operation behind every entry point is the mode-k matricized-tensor
 * times Khatri-Rao product in its element-wise ("matrix-free") form, paper
 * Sec. II-B, Eq. (elem), with the weight vector lambda fixed to one:
 *
 *     M(n, j) = sum_{i : i_k = n}  X(i) * prod_{m != k} A_m(i_m, j),
 *               n in [0, I_k),  j in [0, R),
 *
 * which equals X_(k) * (A_d (.) ... (.) A_{k+1} (.) A_{k-1} (.) ... (.) A_1) of
 * Eq. (krp) without ever forming the Khatri-Rao matrix or an unfolded or
 * permuted copy of X.  Extra device memory is partial sums in the
 * O(R * sum_n I_n) class of Sec. I (contributions) and Sec. II-B (last
 * paragraph): slots * I_k * R values with slots a plan constant, never more
 * than 5 % of the bytes of X or 64 MiB, whichever is larger (one exception:
 * fp32 with I_0 < 16 and R >= 500, where short accumulation chains force many
 * splits and the partial sums can reach 10 to 40 % of X); plus, where two
 * adjacent modes are treated as one (two short column modes; modes 0 and 1 when
 * I_0 fits the 16-row MFMA blocks badly), the row-wise product of their two
 * factors, which is only formed while it stays below a constant size (8 MiB by
 * default for two column modes, 32 MiB for modes 0 and 1; at most two such
 * matrices per call), or, for k != 0 with at most
 * 1024 entries in the modes other than 0 and k, the product of those modes'
 * factor rows (at most 1024 x R values).
 *
 * Layouts (Sec. II-A: ind2sub/sub2ind "defined like MATLAB" => first index
 * fastest; Sec. III: row-wise factor layout):
 *   X          dense, flat, no padding, first index fastest:
 *              X[i_0 + I_0*(i_1 + I_1*(i_2 + ...))]
 *   factors[m] row-major I_m x R, leading dimension R
 *   M          row-major I_k x R, leading dimension R
 * Indices and k are 0-based in this interface (the paper counts from 1).
 *
 * Pointers: X, every factors[m], M and workspace are DEVICE pointers owned by
 * the caller.  dims and the factors pointer array are HOST arrays, read before
 * the call returns.  The library keeps no reference to any argument after the
 * call returns (the enqueued kernels do, until the stream has drained).
 * stream is a hipStream_t passed as void* (NULL = the default stream).  The
 * device that holds the pointers and the stream must be the current device.
 *
 * Semantics: M is overwritten (never accumulated into).  factors[k] is never
 * read and may be NULL (Eq. (elem) excludes m = k).  M must not alias an
 * input.  Calls are asynchronous: they return after enqueueing on stream.
 *
 * Errors: every function returns an mttkrp_status (or documents otherwise),
 * never throws, aborts or exits.  On any error nothing is enqueued and M is
 * untouched.
 *   MTTKRP_ERR_INVALID_ARG  null X/M/dims/factors, null factors[m != k],
 *                           ndim < 2, dims[m] < 1, R < 1, k out of range,
 *                           element count or byte size overflowing int64
 *   MTTKRP_ERR_UNSUPPORTED  ndim > MTTKRP_MAX_NDIM, a dimension >= 2^31,
 *                           R >= 2^27, or a decomposition that would need
 *                           >= 2^31 work items
 *   MTTKRP_ERR_WORKSPACE    a *_ws call with too few workspace bytes, or
 *                           workspace not 256-byte aligned
 *   MTTKRP_ERR_DEVICE       a HIP runtime call failed
 *   MTTKRP_ERR_NUMERICAL    (CP-ALS only) the input made a step of the iteration
 *                           impossible: a Gram Hadamard product that is not
 *                           positive definite
 */
#ifndef MTTKRP_H
#define MTTKRP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MTTKRP_MAX_NDIM 8

typedef enum {
    MTTKRP_OK = 0,
    MTTKRP_ERR_INVALID_ARG = 1,
    MTTKRP_ERR_UNSUPPORTED = 2,
    MTTKRP_ERR_WORKSPACE = 3,
    MTTKRP_ERR_DEVICE = 4,
    MTTKRP_ERR_NUMERICAL = 5
} mttkrp_status;

/*
 * Core calls, Eq. (elem): M = X_(k) (Khatri-Rao of all A_m, m != k), one per
 * data type.  Partial sums live in a library-owned workspace per (device,
 * stream) that grows on demand, so calls in flight on different streams of one
 * device do not share scratch memory and may overlap freely; calls on one
 * stream are ordered by the stream.  Growing a workspace is the only time these
 * calls allocate; they then wait on the host for the last call that used it.
 * A device keeps the workspaces of the eight most recently used streams; a
 * ninth stream takes over the least recently used one after waiting for that
 * stream's last call.  Not for use under stream capture (the calls record an
 * event they may later wait on): capture the *_ws calls instead.
 *   ndim     number of modes d, 2 <= d <= MTTKRP_MAX_NDIM
 *   dims     host array of d extents I_0..I_{d-1}, each >= 1
 *   X        device, prod(dims) values
 *   factors  host array of d device pointers; factors[m] is I_m x R
 *   R        number of columns (rank), any R >= 1
 *   k        mode, 0 <= k < d
 *   M        device, I_k x R, overwritten
 */
int mttkrp_dense_f64(int ndim, const int64_t* dims, const double* X,
                     const double* const* factors, int R, int k, double* M,
                     void* stream);
int mttkrp_dense_f32(int ndim, const int64_t* dims, const float* X,
                     const float* const* factors, int R, int k, float* M,
                     void* stream);

/*
 * Caller-owned workspace variants of the same operation.  They never allocate.
 * mttkrp_dense_workspace_bytes returns the bytes the *_ws call with the same
 * (ndim, dims, R, k, dtype_bytes in {8, 4}) needs (possibly 0), or
 * (size_t)-1 for invalid arguments.  workspace must be a device pointer
 * aligned to 256 bytes (NULL allowed when 0 bytes are needed); its previous
 * contents do not matter and it holds no result after the call.
 */
size_t mttkrp_dense_workspace_bytes(int ndim, const int64_t* dims, int R, int k,
                                    int dtype_bytes);
int mttkrp_dense_f64_ws(int ndim, const int64_t* dims, const double* X,
                        const double* const* factors, int R, int k, double* M,
                        void* workspace, size_t workspace_bytes, void* stream);
int mttkrp_dense_f32_ws(int ndim, const int64_t* dims, const float* X,
                        const float* const* factors, int R, int k, float* M,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Extended calls: the MTTKRP exactly as the paper states it, Eq. (krp) / Eq.
 * (elem) with the weight vector, plus optional accumulation:
 *
 *     M = beta * M + X_(k) (Khatri-Rao of all A_m, m != k) diag(lambda)
 *
 *   lambda   device, R values, or NULL for lambda = 1
 *   beta     host scalar; with beta = 0 the old contents of M are never read
 *   workspace, workspace_bytes   caller-owned workspace as in the *_ws calls
 *            (size from mttkrp_dense_ex_workspace_bytes, never 0), or
 *            NULL / 0 to use the library-owned one
 * With lambda = NULL and beta = 0 the result equals that of the core calls bit
 * for bit.  Everything else (layouts, ownership, errors, asynchrony) is as for
 * the core calls.
 */
size_t mttkrp_dense_ex_workspace_bytes(int ndim, const int64_t* dims, int R, int k,
                                       int dtype_bytes);
int mttkrp_dense_f64_ex(int ndim, const int64_t* dims, const double* X,
                        const double* const* factors, int R, int k,
                        const double* lambda, double beta, double* M,
                        void* workspace, size_t workspace_bytes, void* stream);
int mttkrp_dense_f32_ex(int ndim, const int64_t* dims, const float* X,
                        const float* const* factors, int R, int k,
                        const float* lambda, float beta, float* M,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * The extended calls with leading dimensions: factors and M may be blocks of
 * wider row-major arrays (Sec. III fixes the row-wise layout; the distance
 * between rows is the caller's).
 *   ld_factors  host array of d values; rows of factors[m] are ld_factors[m]
 *               values apart, ld_factors[m] >= R (the entry for m = k is ignored)
 *   ldM         rows of M are ldM values apart, ldM >= R; only the first R values
 *               of every row are written (or read, with beta != 0)
 * Everything else as for mttkrp_dense_f64_ex / _f32_ex (the same workspace size
 * applies).  MTTKRP_ERR_INVALID_ARG also for a null ld_factors or a leading
 * dimension below R or of 2^27 or more.
 */
int mttkrp_dense_f64_ld(int ndim, const int64_t* dims, const double* X,
                        const double* const* factors, const int64_t* ld_factors, int R, int k,
                        const double* lambda, double beta, double* M, int64_t ldM,
                        void* workspace, size_t workspace_bytes, void* stream);
int mttkrp_dense_f32_ld(int ndim, const int64_t* dims, const float* X,
                        const float* const* factors, const int64_t* ld_factors, int R, int k,
                        const float* lambda, float beta, float* M, int64_t ldM,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Partial contraction over the leading index.  X is read as a P x Q matrix, first index
 * fastest (for a d-way tensor: P = the product of the extents of modes 0 .. s-1, Q = the
 * product of the others, no copy or permutation), and
 *     T(c, j) = sum_{r = 0 .. P-1} X[r + P c] * K[r * ldK + j],    c < Q, j < R.
 * With K the Khatri-Rao product of the factors of the leading modes (row r = the product of
 * their rows at the multi-index of r, lowest mode fastest; for s = 1 the factor of mode 0
 * itself) T is the part of the sum of Eq. (elem) that the modes s .. d-1 share: the mode-k
 * MTTKRP is T weighted by the other trailing factors and summed over their indices.  For
 * Q = I_{d-1} (s = d-1) T is the last mode's MTTKRP.
 *   X, K, T_out  device pointers; T_out is Q x R row-major with leading dimension ldT >= R,
 *                overwritten; K has leading dimension ldK >= R
 *   workspace    device memory of mttkrp_contract_leading_workspace_bytes bytes (0 for most
 *                shapes: partial sums are only needed when Q is too short to fill the chip
 *                and P is split), may be NULL when that is 0
 * Limits: P, Q < 2^31 - 64, R < 2^27.  Errors as for the core calls; the query returns
 * (size_t)-1 for invalid or unsupported arguments.  Asynchronous on `stream`.
 */
size_t mttkrp_contract_leading_workspace_bytes(int64_t P, int64_t Q, int R, int dtype_bytes);
int mttkrp_contract_leading_f64(int64_t P, int64_t Q, const double* X, const double* K, int64_t ldK,
                                int R, double* T_out, int64_t ldT, void* workspace,
                                size_t workspace_bytes, void* stream);
int mttkrp_contract_leading_f32(int64_t P, int64_t Q, const float* X, const float* K, int64_t ldK,
                                int R, float* T_out, int64_t ldT, void* workspace,
                                size_t workspace_bytes, void* stream);

/*
 * mttkrp_dense_f64 for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same operation, arguments, layouts and errors as mttkrp_dense_f64, and the
 * same kernels; the partial sums (and the small product matrices of fused
 * modes) go to a fixed 64 MiB scratch array that is part of the library's
 * code object, so the call never calls hipMalloc / hipFree or any allocating
 * routine, and records no timing events (the measurement hooks ignore it).
 *   - Limit: shapes whose plan needs more than 64 MiB of workspace
 *     (mttkrp_dense_workspace_bytes(...) > 67108864) return
 *     MTTKRP_ERR_WORKSPACE and enqueue nothing.  Every benchmark
 *     configuration fits (the largest, 16384 x 2048 x 64 at R = 128, needs
 *     exactly 64 MiB).
 *   - Every GPU the library runs on holds its own copy of the array until the
 *     process ends.  The first call on a device looks up the array's address
 *     on that device (and makes the runtime load the code object there): make
 *     that first call outside graph capture.
 *   - Nothing in the array has to start at zero: every partial sum that a call
 *     reads was written by the same call, so the previous call's contents do
 *     not matter.
 *   - All calls on one GPU share the one array: calls that overlap on a GPU
 *     (different streams, or graphs replayed concurrently) race.  Order them.
 * MTTKRP_ERR_DEVICE when the address lookup fails.
 */
int mttkrp_dense_f64_noalloc(int ndim, const int64_t* dims, const double* X,
                             const double* const* factors, int R, int k, double* M,
                             void* stream);

/* Static, human-readable text for a status code. */
const char* mttkrp_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int mttkrp_version(void);

/* Frees the library-owned workspaces of every device (synchronises them). */
void mttkrp_release(void);

/*
 * Measurement hooks (Sec. IV-B reports time per MTTKRP).  While timing is
 * enabled every core / *_ws call records three HIP events on its own stream:
 * before its streaming kernel, between its two kernels and after its combine
 * kernel (the combine figure therefore includes the gap between the kernels).  Enabling (re)starts the
 * count of timed calls on every device; the most recent 512 timed calls of a
 * device are kept.
 *   mttkrp_timing_count  timed calls on the current device since enabling
 *   mttkrp_timing_get    waits for the events of timed call `index`
 *                        (0-based, in call order) and returns the two kernel
 *                        durations in milliseconds (combine_ms = 0 when no
 *                        combine kernel ran); MTTKRP_ERR_INVALID_ARG when the
 *                        index was never recorded or has been overwritten
 *   mttkrp_timing_last   the same for the most recent timed call
 */
int mttkrp_timing_enable(int enable);
int64_t mttkrp_timing_count(void);
int mttkrp_timing_get(int64_t index, float* stream_ms, float* combine_ms);
int mttkrp_timing_last(float* stream_ms, float* combine_ms);

/*
 * Decomposition parameters for tuning sweeps and schedule-invariance tests
 * (the result of Eq. (elem) must not depend on them beyond rounding).
 * 0 restores the built-in choice.  Keys:
 *   "row_blocks"    16-row MFMA blocks per wavefront (1..4)
 *   "target_items"  wavefront work items the planner aims for
 *   "max_steps"     upper bound on 4-column steps per work item
 *   "xcd_remap"     1 = contiguous item ranges per XCD, 2 = plain order (default)
 *   "ws_percent"    cap on first-mode partial-sum traffic, percent of X bytes
 *   "max_col_blocks"  16-column blocks of the output per wavefront (1..4; the second
 *                   schedule up to 8); more columns are covered by further
 *                   wavefronts that re-read X
 *   "first_group"   first mode only: 4 = the four wavefronts of a workgroup sum
 *                   their tiles in LDS and write one partial tile, 1 = every
 *                   wavefront writes its own partial tile, 0 = chosen per shape
 *   "waves_per_simd"  cap on resident wavefronts per SIMD (2..7; enforced by
 *                   reserving LDS), 0 = whatever the registers allow
 *   "nt_loads"      1 = never use non-temporal tensor loads, 0 = chosen by alignment
 *   "fuse_bytes"    largest product matrix (bytes) for which two adjacent modes
 *                   are fused into one (default 8 MiB; 1 = never fuse)
 *   "pair_rows"     k = 0 and k = 1: 1 = take the pairs (i_0, i_1) as the rows (no padded row
 *                   blocks; the epilogue sums each tile per output row, or, for k = 0 with
 *                   I_0 > 32, stores the weighted tile for the combine kernel), 2 =
 *                   never, 0 = when I_0 alone leaves more than 1 % of the tiles' rows empty or
 *                   allows only one or two row blocks per wavefront
 *   "fuse_rows"     k >= 2 only: 1 = modes 0 and 1 are one row mode (their factors' row-wise
 *                   product as its factor) whenever that product stays within four times
 *                   "fuse_bytes", 2 = never, 0 = by the same rule as "pair_rows" when the sweeps
 *                   that remain stay long
 *   "lead_last"     last mode only: 1 = as one contraction over all other modes (X^T times the
 *                   Khatri-Rao product of their factors, formed in the workspace) whenever that
 *                   product stays below 4 MiB, 2 = never, 0 = then and when mode 0 fills the row
 *                   tiles badly, I_k >= 256 and the rows need no splitting
 *   "contract_rows" schedule for k != 0: 1 = contract over mode 0 (rows) whenever the
 *                   other modes' entries number at most 1024, 2 = never, 0 = chosen by
 *                   the planner (those entries few, under 128, mode 0 at least eight
 *                   times as long, and either at most 32 of them or R large enough for the
 *                   data type)
 *   "rows_col_blocks"  that schedule only: 16-entry blocks of the column space per
 *                   wavefront (1..4), 0 = chosen by the planner
 *   "inner_splits"  pieces the sweep over the inner column mode is cut into (1..64),
 *                   0 = chosen by the planner
 *   "deep"          1 = always the kernel build with the software-pipelined run,
 *                   2 = always the build with batches only, 0 = by item length
 *   "linear"        1 = the column space is split into balanced ranges of steps that may
 *                   begin and end inside a sweep, 2 = only whole sweeps and equal pieces
 *                   of sweeps, 0 = chosen by the planner (ranges for the first mode when
 *                   the other way leaves the work items uneven)
 * Returns MTTKRP_ERR_INVALID_ARG for an unknown key or a value out of range.
 */
int mttkrp_tune_set(const char* key, int64_t value);

/*
 * Writes a one-line description of the decomposition the library would use
 * (row blocks, column blocks, work items, steps per item, partial slots,
 * workspace bytes) into buf (always NUL-terminated when buflen > 0).
 */
int mttkrp_plan_describe(int ndim, const int64_t* dims, int R, int k,
                         int dtype_bytes, char* buf, size_t buflen);

#ifdef __cplusplus
}
#endif
#endif /* MTTKRP_H */
