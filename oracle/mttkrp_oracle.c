/*
 * CPU oracle for the matrix-free dense mode-k MTTKRP.
 *
 * TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  Only the test-suite, the smoke
 * check and the benchmark's CPU-baseline leg may call this file.  It shares no
 * code, header, table or helper with the HIP library and must stay that way.
 *
 * What it computes is the element-wise definition of the MTTKRP (paper
 * Sec. II-B, Eq. (elem)):
 *
 *     M(n, j) = lambda_j * sum over all multi-indices i with i_k = n of
 *               X(i) * prod_{m != k} A_m(i_m, j)
 *
 * with the weight vector lambda optional (NULL means lambda = 1, which is the
 * hot path of the library under test),
 * written out as a plain loop over every tensor entry.  No blocking, no
 * factoring of the product, no re-association beyond "one running sum per
 * output entry, in storage order of X".
 *
 * Layouts (Sec. II-A: MATLAB-like ind2sub/sub2ind => first index fastest;
 * Sec. III: row-wise factor layout):
 *   X        flat, first-index-fastest:  lin(i) = sum_m i_m * prod_{l<m} I_l
 *   A_m      row-major I_m x R, leading dimension R
 *   M        row-major, leading dimension R
 * Indices are 0-based here (the paper is 1-based).
 *
 * Row independence (Sec. III: row n of the result depends only on the mode-k
 * subtensor S_n^(k)) is what makes "one output row at a time" the same sum as
 * one sweep over the whole tensor; OpenMP threads each own whole output rows
 * (or whole column blocks of a row), so the arithmetic per output entry is a
 * single sequential chain regardless of the thread count.
 *
 * Accumulator type:
 *   *_f64 / *_f32            long double (x87 80-bit on x86-64) running sums,
 *                            products formed in long double, rounded once at
 *                            the end.  This is the parity reference.
 *   *_f64_native/_f32_native the same loop with the running sum and products
 *                            in the data type itself (what a plain CPU code
 *                            would do); used for the error-bound pin and as a
 *                            second timed CPU figure.
 *
 * Parity status: pinned (see tests/test_oracle_pins.py): explicit unfolding
 * times explicit Khatri-Rao product, rank-1 and rank-S closed forms, numpy
 * matmul/einsum special cases, linearity, independence from A_k and from
 * entries outside the subtensor, marginals, mode-permutation equivariance.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MAX_NDIM 16

enum {
    ORACLE_OK = 0,
    ORACLE_BAD_ARG = 1,
    ORACLE_NO_MEM = 2
};

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int oracle_long_double_mant_bits(void)
{
    return (int)__LDBL_MANT_DIG__;
}

/* Shared argument checks.  Returns ORACLE_OK or ORACLE_BAD_ARG. */
static int check_args(int ndim, const int64_t *dims, const void *X,
                      const void *const *factors, int R, int k,
                      const int64_t *rows, int64_t nrows, const void *M)
{
    if (ndim < 1 || ndim > ORACLE_MAX_NDIM || !dims || !X || !factors || !M)
        return ORACLE_BAD_ARG;
    if (R < 1 || k < 0 || k >= ndim)
        return ORACLE_BAD_ARG;
    for (int m = 0; m < ndim; ++m) {
        if (dims[m] < 1)
            return ORACLE_BAD_ARG;
        if (m != k && !factors[m])
            return ORACLE_BAD_ARG;
    }
    if (rows) {
        if (nrows < 0)
            return ORACLE_BAD_ARG;
        for (int64_t t = 0; t < nrows; ++t)
            if (rows[t] < 0 || rows[t] >= dims[k])
                return ORACLE_BAD_ARG;
    }
    return ORACLE_OK;
}

/*
 * One generic body, instantiated four times.
 *   T    data type of X, the factors and M
 *   ACC  type of products and running sums
 *
 * Work item w = (t, jb): output row number t of the request (row index
 * n = rows[t], or t itself when rows == NULL) and column block jb.  Column
 * blocks exist only so that a mode with fewer rows than threads still keeps
 * every thread busy; each (n, j) entry is still one sequential chain.
 */
#define DEFINE_ORACLE(NAME, T, ACC)                                            \
int NAME(int ndim, const int64_t *dims, const T *X,                            \
         const T *const *factors, int R, int k,                                \
         const int64_t *rows, int64_t nrows, const T *lambda, T *M)            \
{                                                                              \
    int rc = check_args(ndim, dims, X, (const void *const *)factors, R, k,     \
                        rows, nrows, M);                                       \
    if (rc != ORACLE_OK)                                                       \
        return rc;                                                             \
    if (!rows)                                                                 \
        nrows = dims[k];                                                       \
    int64_t stride[ORACLE_MAX_NDIM];                                           \
    int64_t sub_count = 1; /* N_S = N / I_k */                                 \
    {                                                                          \
        int64_t s = 1;                                                         \
        for (int m = 0; m < ndim; ++m) {                                       \
            stride[m] = s;                                                     \
            s *= dims[m];                                                      \
            if (m != k)                                                        \
                sub_count *= dims[m];                                          \
        }                                                                      \
    }                                                                          \
    int nthreads = oracle_max_threads();                                       \
    int64_t jblocks = 1;                                                       \
    if (nrows < nthreads && nrows > 0) {                                       \
        jblocks = (nthreads + nrows - 1) / nrows;                              \
        if (jblocks > R)                                                       \
            jblocks = R;                                                       \
    }                                                                          \
    int64_t jchunk = (R + jblocks - 1) / jblocks;                              \
    int64_t nitems = nrows * jblocks;                                          \
    int failed = 0;                                                            \
    _Pragma("omp parallel for schedule(dynamic, 1)")                           \
    for (int64_t w = 0; w < nitems; ++w) {                                     \
        int64_t t = w / jblocks;                                               \
        int64_t j0 = (w % jblocks) * jchunk;                                   \
        int64_t j1 = j0 + jchunk < R ? j0 + jchunk : R;                        \
        if (j0 >= j1)                                                          \
            continue;                                                          \
        int64_t n = rows ? rows[t] : t;                                        \
        ACC *acc = (ACC *)calloc((size_t)(j1 - j0), sizeof(ACC));              \
        if (!acc) {                                                            \
            _Pragma("omp atomic write")                                        \
            failed = 1;                                                        \
            continue;                                                          \
        }                                                                      \
        /* odometer over the subtensor S_n^(k): every mode but k, lowest     */\
        /* mode fastest, which is also increasing storage order of X.        */\
        int64_t idx[ORACLE_MAX_NDIM];                                          \
        for (int m = 0; m < ndim; ++m)                                         \
            idx[m] = 0;                                                        \
        idx[k] = n;                                                            \
        int64_t lin = n * stride[k];                                           \
        for (int64_t e = 0; e < sub_count; ++e) {                              \
            ACC x = (ACC)X[lin];                                               \
            for (int64_t j = j0; j < j1; ++j) {                                \
                ACC p = x;                                                     \
                for (int m = 0; m < ndim; ++m)                                 \
                    if (m != k)                                                \
                        p *= (ACC)factors[m][idx[m] * (int64_t)R + j];         \
                acc[j - j0] += p;                                              \
            }                                                                  \
            /* advance the odometer */                                         \
            for (int m = 0; m < ndim; ++m) {                                   \
                if (m == k)                                                    \
                    continue;                                                  \
                idx[m] += 1;                                                   \
                lin += stride[m];                                              \
                if (idx[m] < dims[m])                                          \
                    break;                                                     \
                lin -= idx[m] * stride[m];                                     \
                idx[m] = 0;                                                    \
            }                                                                  \
        }                                                                      \
        for (int64_t j = j0; j < j1; ++j) {                                    \
            ACC v = acc[j - j0];                                               \
            if (lambda)                                                        \
                v = (ACC)lambda[j] * v;                                        \
            M[t * (int64_t)R + j] = (T)v;                                      \
        }                                                                      \
        free(acc);                                                             \
    }                                                                          \
    return failed ? ORACLE_NO_MEM : ORACLE_OK;                                 \
}

DEFINE_ORACLE(oracle_mttkrp_f64, double, long double)
DEFINE_ORACLE(oracle_mttkrp_f32, float, long double)
DEFINE_ORACLE(oracle_mttkrp_f64_native, double, double)
DEFINE_ORACLE(oracle_mttkrp_f32_native, float, float)
