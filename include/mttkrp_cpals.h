/*
 * mttkrp_cpals.h -- a minimal CP-ALS driver on top of the dense MTTKRP, and the
 * all-modes sweep it is built from.
 *
 * The paper motivates the MTTKRP as the bottleneck kernel of CP algorithms
 * (Sec. I) and times CP-ALS "with tolerance 1e-4" (Sec. IV-C); it does not
 * print the iteration.  This driver is the textbook alternating least squares
 * for the CP model of Sec. II-A, X ~ sum_j lambda_j a_j^(1) o ... o a_j^(d):
 *
 *   every sweep, for k = 0 .. d-1:
 *       M   = X_(k) (Khatri-Rao of all A_m, m != k)        mttkrp_dense_f64
 *       V   = Hadamard product of the Gram matrices A_m^T A_m, m != k
 *       A_k = M V^{-1}                                      (V = L L^T, two triangular solves)
 *       lambda_j = ||A_k(:, j)||_2,  A_k(:, j) /= lambda_j  (a zero column is left alone)
 *   after the last mode:
 *       fit = 1 - sqrt(max(||X||^2 + ||X^||^2 - 2 <X, X^>, 0)) / ||X||,
 *       <X, X^> = sum_j lambda_j sum_i M(i, j) A_{d-1}(i, j),
 *       ||X^||^2 = lambda^T (Hadamard product of all Gram matrices) lambda
 *   stop when |fit - previous fit| < tol, or after max_iters sweeps.
 *
 * The paper's CP-ALS experiment (Sec. IV-C) runs ranks 10, 500, 1000 and 2000; up to rank
 * 64 the R x R work (Gram matrices, Cholesky factor, row solves) runs in one workgroup's
 * LDS, above that blocked from global memory, 32 columns at a time (then also every
 * I_n <= 1048560).
 *
 * Everything runs on the GPU in fp64 with fixed-order reductions (reruns are
 * bit-identical); the host only reads three scalars per sweep to evaluate the
 * stopping rule.  Layouts, index base and pointer ownership are those of
 * mttkrp.h.  The driver allocates its own device buffers (O(R * max_n I_n +
 * d * R^2) values besides the MTTKRP workspace) and frees them before it
 * returns; it synchronises the stream once per sweep.
 */
#ifndef MTTKRP_CPALS_H
#define MTTKRP_CPALS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MTTKRP_CPALS_MAX_RANK 2048

/*
 * All-modes sweep: M_out[k] = X_(k) (Khatri-Rao of all factors but the k-th)
 * for every k, i.e. d calls of mttkrp_dense_f64 / _f32 on the same resident X
 * (no intermediate is shared between the modes).
 *   M_out   host array of d device pointers, M_out[k] is I_k x R, overwritten
 *   other arguments as mttkrp_dense_*; here every factors[m] is read.
 */
int mttkrp_dense_all_modes_f64(int ndim, const int64_t* dims, const double* X,
                               const double* const* factors, int R, double* const* M_out,
                               void* stream);
int mttkrp_dense_all_modes_f32(int ndim, const int64_t* dims, const float* X,
                               const float* const* factors, int R, float* const* M_out,
                               void* stream);

/*
 * All-modes sweep that shares partial contractions between the modes: the same d results
 * from two passes over X instead of d.  The modes are cut into a leading set 0 .. s-1
 * (P_L = their extents' product) and a trailing set s .. d-1 (P_R); one pass contracts the
 * trailing modes (an MTTKRP of X seen as a P_L x I_s x ... tensor, first mode), one the
 * leading modes (mttkrp_contract_leading_* with the Khatri-Rao product of the leading
 * factors); every mode's result then follows from one of the two intermediates (P_L x R and
 * P_R x R values) by a small kernel.  The sums of Eq. (elem) are the same, taken in another
 * order.  This trades memory for passes: the intermediates are in the class of the partial
 * Khatri-Rao matrices of the paper's Table I, not in O(R sum I_n); the cut with the smallest
 * intermediates is taken, and the call is only supported when everything fits an eighth of
 * the tensor's bytes (or 64 MiB).
 *   mttkrp_dense_all_modes_shared_bytes   bytes of `workspace` the call needs, 0 when the
 *                                         shape is not supported (use mttkrp_dense_all_modes_*)
 *   workspace   device memory, caller-owned, 256-byte aligned; contents need not be kept
 *   other arguments as mttkrp_dense_all_modes_*; M_out[k] may be one buffer for all k only
 *   if the caller consumes each result in stream order (the CP-ALS driver does).
 * Returns MTTKRP_ERR_UNSUPPORTED for a shape without a cut that fits, MTTKRP_ERR_WORKSPACE
 * for a workspace that is too small.  Everything the call needs, the partial sums of the
 * core call of its first pass included, lies in `workspace`: it only enqueues kernels
 * (no allocation, no memset, no copy), so it may be recorded into a HIP graph.  The byte
 * count depends on the decomposition parameters (mttkrp_tune_set) in force at the query.
 */
size_t mttkrp_dense_all_modes_shared_bytes(int ndim, const int64_t* dims, int R, int dtype_bytes);
int mttkrp_dense_all_modes_shared_f64(int ndim, const int64_t* dims, const double* X,
                                      const double* const* factors, int R, double* const* M_out,
                                      void* workspace, size_t workspace_bytes, void* stream);
int mttkrp_dense_all_modes_shared_f32(int ndim, const int64_t* dims, const float* X,
                                      const float* const* factors, int R, float* const* M_out,
                                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * CP-ALS in fp64.
 *   factors    host array of d device pointers; factors[m] is I_m x R: the
 *              initial guess on entry, the column-normalised factor on return
 *   lambda     device, R values, written: the weights
 *   R          1 <= R <= MTTKRP_CPALS_MAX_RANK
 *   max_iters  >= 1 sweeps at most
 *   tol        stop when the fit changes by less than this (0: run max_iters)
 *   iters      host, written: sweeps done
 *   fits       host array of max_iters doubles (or NULL), fits[s] = fit after sweep s
 * Returns an mttkrp_status: MTTKRP_ERR_UNSUPPORTED for R above the limit,
 * MTTKRP_ERR_DEVICE when an allocation or a HIP call fails; MTTKRP_ERR_NUMERICAL
 * when a Gram Hadamard product is not positive definite (its Cholesky factor would
 * hold a non-positive pivot; the factors and lambda then hold the last completed
 * update).
 */
int mttkrp_cpals_f64(int ndim, const int64_t* dims, const double* X, double* const* factors,
                     double* lambda, int R, int max_iters, double tol, int* iters, double* fits,
                     void* stream);

/*
 * The same iteration with every sweep done as in mttkrp_dense_all_modes_shared_f64 (factor k
 * is updated right after its MTTKRP, so later modes see it exactly as in the plain driver;
 * the intermediate of the trailing modes is formed before the leading factors change and
 * does not contain them).  The driver allocates the intermediates' buffer itself; for a
 * shape without a supported cut it runs the plain sweeps.  Results agree with
 * mttkrp_cpals_f64 to rounding (the sums are taken in another order).
 */
int mttkrp_cpals_shared_f64(int ndim, const int64_t* dims, const double* X, double* const* factors,
                            double* lambda, int R, int max_iters, double tol, int* iters,
                            double* fits, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MTTKRP_CPALS_H */
