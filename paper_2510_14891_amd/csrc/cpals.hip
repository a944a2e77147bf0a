// Minimal CP-ALS driver and all-modes sweep on top of the dense MTTKRP.
// C ABI, the iteration and its conventions: include/mttkrp_cpals.h.  Everything
// but the MTTKRP itself is small (R x R or I_k x R) and runs in plain fp64 HIP
// kernels with fixed-order reductions.
#include <hip/hip_runtime.h>

#include <math.h>
#include <stdint.h>

#include "../../include/mttkrp.h"
#include "../../include/mttkrp_cpals.h"

namespace {

constexpr int kChunkRows = 64;     // rows of a factor one workgroup turns into a partial Gram matrix
constexpr int kNormBlocks = 2048;  // partial sums of ||X||^2

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Sum of 256 per-thread values in a fixed tree order; result in every thread.
__device__ __forceinline__ double block_sum_256(double v, double* lds)
{
    lds[threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s)
            lds[threadIdx.x] += lds[threadIdx.x + s];
        __syncthreads();
    }
    const double r = lds[0];
    __syncthreads();
    return r;
}

// partial[b] = sum of squares of block b's contiguous share of X (fixed assignment and order).
__global__ void __launch_bounds__(256) sumsq_partial(const double* __restrict__ X, int64_t N, double* partial)
{
    __shared__ double lds[256];
    const int64_t per = (N + gridDim.x - 1) / gridDim.x;
    const int64_t lo = per * blockIdx.x;
    const int64_t hi = lo + per < N ? lo + per : N;
    double s = 0.0;
    for (int64_t i = lo + threadIdx.x; i < hi; i += 256) {
        const double v = X[i];
        s += v * v;
    }
    s = block_sum_256(s, lds);
    if (threadIdx.x == 0)
        partial[blockIdx.x] = s;
}

// out[0] = sum of n values, one workgroup, fixed order.
__global__ void __launch_bounds__(256) sum_fixed(const double* __restrict__ v, int n, double* out)
{
    __shared__ double lds[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += 256)
        s += v[i];
    s = block_sum_256(s, lds);
    if (threadIdx.x == 0)
        out[0] = s;
}

// Partial Gram matrix of rows [64 b, 64 b + 64) of A (I x R): ws[b][a * R + c] = sum_r A(r, a) A(r, c).
__global__ void __launch_bounds__(256) gram_partial(const double* __restrict__ A, int64_t I, int R, double* ws)
{
    extern __shared__ double tile[];   // kChunkRows x R
    const int64_t r0 = (int64_t)blockIdx.x * kChunkRows;
    const int rows = (int)(I - r0 < kChunkRows ? I - r0 : kChunkRows);
    for (int t = threadIdx.x; t < rows * R; t += 256)
        tile[t] = A[r0 * R + t];
    __syncthreads();
    double* out = ws + (int64_t)blockIdx.x * R * R;
    for (int e = threadIdx.x; e < R * R; e += 256) {
        const int a = e / R, c = e - a * R;
        double s = 0.0;
        for (int r = 0; r < rows; ++r)
            s += tile[r * R + a] * tile[r * R + c];
        out[e] = s;
    }
}

// G[e] = sum over chunks of ws[chunk][e], in chunk order.
__global__ void __launch_bounds__(256) gram_reduce(const double* __restrict__ ws, int n_chunks, int RR, double* G)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= RR)
        return;
    double s = 0.0;
    for (int c = 0; c < n_chunks; ++c)
        s += ws[(int64_t)c * RR + e];
    G[e] = s;
}

// V = Hadamard product of the Gram matrices of all modes but `skip` (skip < 0: of all modes).
__global__ void __launch_bounds__(256) hadamard_grams(const double* __restrict__ G, int ndim, int RR, int skip, double* V)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= RR)
        return;
    double v = 1.0;
    for (int m = 0; m < ndim; ++m)
        if (m != skip)
            v *= G[(int64_t)m * RR + e];
    V[e] = v;
}

// In-place Cholesky factor of the R x R matrix V (lower triangle, L L^T = V) by one workgroup.
// flag[0] is set to 1 when a pivot is not positive.
__global__ void __launch_bounds__(256) cholesky_lower(double* V, int R, int* flag)
{
    extern __shared__ double Ls[];   // R x R
    for (int t = threadIdx.x; t < R * R; t += 256)
        Ls[t] = V[t];
    __syncthreads();
    for (int j = 0; j < R; ++j) {
        const double piv = Ls[j * R + j];
        if (!(piv > 0.0)) {
            if (threadIdx.x == 0)
                flag[0] = 1;
            return;   // uniform: every thread sees the same pivot
        }
        const double dj = sqrt(piv);
        __syncthreads();
        for (int i = j + threadIdx.x; i < R; i += 256)
            Ls[i * R + j] = i == j ? dj : Ls[i * R + j] / dj;
        __syncthreads();
        const int n = R - j - 1;
        for (int t = threadIdx.x; t < n * n; t += 256) {
            const int i = j + 1 + t / n, c = j + 1 + t % n;
            if (c <= i)
                Ls[i * R + c] -= Ls[i * R + j] * Ls[c * R + j];
        }
        __syncthreads();
    }
    for (int t = threadIdx.x; t < R * R; t += 256) {
        const int i = t / R, c = t - i * R;
        V[t] = c <= i ? Ls[t] : 0.0;
    }
}

// Rows of A = M V^{-1} with V = L L^T: forward solve L y = m, backward solve L^T z = y, one
// thread per row, 32 rows per workgroup; L and the rows live in LDS.
__global__ void __launch_bounds__(32) solve_rows(const double* __restrict__ L, const double* __restrict__ M,
                                                  int64_t I, int R, double* A, const int* flag)
{
    extern __shared__ double lds[];
    if (flag[0])      // no valid factor: leave A_k as it is
        return;
    double* Ls = lds;                       // R x R
    double* Y = lds + R * R;                // 32 x (R + 1)
    for (int t = threadIdx.x; t < R * R; t += 32)
        Ls[t] = L[t];
    const int64_t row = (int64_t)blockIdx.x * 32 + threadIdx.x;
    double* y = Y + threadIdx.x * (R + 1);
    if (row < I)
        for (int a = 0; a < R; ++a)
            y[a] = M[row * R + a];
    __syncthreads();
    if (row >= I)
        return;
    for (int a = 0; a < R; ++a) {
        double s = y[a];
        for (int b = 0; b < a; ++b)
            s -= Ls[a * R + b] * y[b];
        y[a] = s / Ls[a * R + a];
    }
    for (int a = R - 1; a >= 0; --a) {
        double s = y[a];
        for (int b = a + 1; b < R; ++b)
            s -= Ls[b * R + a] * y[b];
        y[a] = s / Ls[a * R + a];
    }
    for (int a = 0; a < R; ++a)
        A[row * R + a] = y[a];
}

// Workgroup j: lambda[j] = 2-norm of column j of A (I x R), then the column is divided by it.
__global__ void __launch_bounds__(256) normalise_columns(double* A, int64_t I, int R, double* lambda, const int* flag)
{
    __shared__ double lds[256];
    if (flag[0])
        return;
    const int j = blockIdx.x;
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < I; i += 256) {
        const double v = A[i * R + j];
        s += v * v;
    }
    s = block_sum_256(s, lds);
    const double nrm = sqrt(s);
    if (threadIdx.x == 0)
        lambda[j] = nrm;
    if (nrm > 0.0)
        for (int64_t i = threadIdx.x; i < I; i += 256)
            A[i * R + j] /= nrm;
}

// Workgroup j: col[j] = lambda[j] * sum_i M(i, j) A(i, j).
__global__ void __launch_bounds__(256) inner_product_columns(const double* __restrict__ M, const double* __restrict__ A,
                                                              const double* __restrict__ lambda, int64_t I, int R,
                                                              double* col)
{
    __shared__ double lds[256];
    const int j = blockIdx.x;
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < I; i += 256)
        s += M[i * R + j] * A[i * R + j];
    s = block_sum_256(s, lds);
    if (threadIdx.x == 0)
        col[j] = lambda[j] * s;
}

// out[0] = lambda^T V lambda, one workgroup, fixed order (row sums, then their sum).
__global__ void __launch_bounds__(256) quadratic_form(const double* __restrict__ V, const double* __restrict__ lambda,
                                                       int R, double* out)
{
    __shared__ double lds[256];
    double s = 0.0;
    for (int a = threadIdx.x; a < R; a += 256) {
        double r = 0.0;
        for (int c = 0; c < R; ++c)
            r += V[a * R + c] * lambda[c];
        s += lambda[a] * r;
    }
    s = block_sum_256(s, lds);
    if (threadIdx.x == 0)
        out[0] = s;
}

struct Buffers {
    double* M = nullptr;        // max_n I_n x R
    double* G = nullptr;        // d x R x R Gram matrices
    double* V = nullptr;        // R x R
    double* gram_ws = nullptr;  // chunks x R x R
    double* partial = nullptr;  // kNormBlocks + R values
    double* scalars = nullptr;  // ||X||^2, <X, X^>, ||X^||^2
    int* flag = nullptr;
    ~Buffers()
    {
        (void)hipFree(M); (void)hipFree(G); (void)hipFree(V); (void)hipFree(gram_ws);
        (void)hipFree(partial); (void)hipFree(scalars); (void)hipFree(flag);
    }
};

void gram(const double* A, int64_t I, int R, double* ws, double* G, hipStream_t st)
{
    const int n_chunks = (int)ceil_div(I, kChunkRows);
    hipLaunchKernelGGL(gram_partial, dim3(n_chunks), dim3(256), (size_t)kChunkRows * R * sizeof(double), st, A, I, R, ws);
    hipLaunchKernelGGL(gram_reduce, dim3((unsigned)ceil_div(R * R, 256)), dim3(256), 0, st, ws, n_chunks, R * R, G);
}

}  // namespace

extern "C" {

int mttkrp_dense_all_modes_f64(int ndim, const int64_t* dims, const double* X, const double* const* factors,
                               int R, double* const* M_out, void* stream)
{
    if (!M_out || ndim < 2 || ndim > MTTKRP_MAX_NDIM)
        return !M_out || ndim < 2 ? MTTKRP_ERR_INVALID_ARG : MTTKRP_ERR_UNSUPPORTED;
    for (int k = 0; k < ndim; ++k) {
        const int rc = mttkrp_dense_f64(ndim, dims, X, factors, R, k, M_out[k], stream);
        if (rc != MTTKRP_OK)
            return rc;
    }
    return MTTKRP_OK;
}

int mttkrp_dense_all_modes_f32(int ndim, const int64_t* dims, const float* X, const float* const* factors,
                               int R, float* const* M_out, void* stream)
{
    if (!M_out || ndim < 2 || ndim > MTTKRP_MAX_NDIM)
        return !M_out || ndim < 2 ? MTTKRP_ERR_INVALID_ARG : MTTKRP_ERR_UNSUPPORTED;
    for (int k = 0; k < ndim; ++k) {
        const int rc = mttkrp_dense_f32(ndim, dims, X, factors, R, k, M_out[k], stream);
        if (rc != MTTKRP_OK)
            return rc;
    }
    return MTTKRP_OK;
}

int mttkrp_cpals_f64(int ndim, const int64_t* dims, const double* X, double* const* factors, double* lambda,
                     int R, int max_iters, double tol, int* iters, double* fits, void* stream)
{
    if (!dims || !X || !factors || !lambda || !iters || ndim < 2 || R < 1 || max_iters < 1 || !(tol >= 0.0))
        return MTTKRP_ERR_INVALID_ARG;
    if (ndim > MTTKRP_MAX_NDIM || R > MTTKRP_CPALS_MAX_RANK)
        return MTTKRP_ERR_UNSUPPORTED;
    int64_t N = 1, max_I = 1;
    for (int m = 0; m < ndim; ++m) {
        if (dims[m] < 1 || !factors[m])
            return MTTKRP_ERR_INVALID_ARG;
        if (dims[m] >= ((int64_t)1 << 31))
            return MTTKRP_ERR_UNSUPPORTED;
        if (N > ((int64_t)1 << 57) / dims[m])
            return MTTKRP_ERR_INVALID_ARG;
        N *= dims[m];
        if (dims[m] > max_I)
            max_I = dims[m];
    }
    *iters = 0;
    hipStream_t st = (hipStream_t)stream;
    const int RR = R * R;
    Buffers b;
    const int64_t max_chunks = ceil_div(max_I, kChunkRows);
    if (hipMalloc(&b.M, (size_t)max_I * R * sizeof(double)) != hipSuccess ||
        hipMalloc(&b.G, (size_t)ndim * RR * sizeof(double)) != hipSuccess ||
        hipMalloc(&b.V, (size_t)RR * sizeof(double)) != hipSuccess ||
        hipMalloc(&b.gram_ws, (size_t)max_chunks * RR * sizeof(double)) != hipSuccess ||
        hipMalloc(&b.partial, (size_t)(kNormBlocks + R) * sizeof(double)) != hipSuccess ||
        hipMalloc(&b.scalars, 3 * sizeof(double)) != hipSuccess ||
        hipMalloc(&b.flag, sizeof(int)) != hipSuccess)
        return MTTKRP_ERR_DEVICE;

    // ||X||^2 once, Gram matrices of the initial factors, cleared pivot flag
    const int nb = (int)(N < kNormBlocks ? N : kNormBlocks);
    hipLaunchKernelGGL(sumsq_partial, dim3(nb), dim3(256), 0, st, X, N, b.partial);
    hipLaunchKernelGGL(sum_fixed, dim3(1), dim3(256), 0, st, b.partial, nb, b.scalars + 0);
    for (int m = 0; m < ndim; ++m)
        gram(factors[m], dims[m], R, b.gram_ws, b.G + (int64_t)m * RR, st);
    int zero = 0;
    if (hipMemcpyAsync(b.flag, &zero, sizeof(int), hipMemcpyHostToDevice, st) != hipSuccess)
        return MTTKRP_ERR_DEVICE;

    const double* cf[MTTKRP_MAX_NDIM];
    double fit_prev = 0.0;
    for (int sweep = 0; sweep < max_iters; ++sweep) {
        for (int k = 0; k < ndim; ++k) {
            for (int m = 0; m < ndim; ++m)
                cf[m] = factors[m];
            const int rc = mttkrp_dense_f64(ndim, dims, X, cf, R, k, b.M, stream);
            if (rc != MTTKRP_OK)
                return rc;
            hipLaunchKernelGGL(hadamard_grams, dim3((unsigned)ceil_div(RR, 256)), dim3(256), 0, st, b.G, ndim, RR, k, b.V);
            hipLaunchKernelGGL(cholesky_lower, dim3(1), dim3(256), (size_t)RR * sizeof(double), st, b.V, R, b.flag);
            hipLaunchKernelGGL(solve_rows, dim3((unsigned)ceil_div(dims[k], 32)), dim3(32),
                               (size_t)(RR + 32 * (R + 1)) * sizeof(double), st, b.V, b.M, dims[k], R, factors[k], b.flag);
            hipLaunchKernelGGL(normalise_columns, dim3(R), dim3(256), 0, st, factors[k], dims[k], R, lambda, b.flag);
            gram(factors[k], dims[k], R, b.gram_ws, b.G + (int64_t)k * RR, st);
        }
        // fit terms: b.M still holds the last mode's MTTKRP
        hipLaunchKernelGGL(inner_product_columns, dim3(R), dim3(256), 0, st, b.M, factors[ndim - 1], lambda,
                           dims[ndim - 1], R, b.partial + kNormBlocks);
        hipLaunchKernelGGL(sum_fixed, dim3(1), dim3(256), 0, st, b.partial + kNormBlocks, R, b.scalars + 1);
        hipLaunchKernelGGL(hadamard_grams, dim3((unsigned)ceil_div(RR, 256)), dim3(256), 0, st, b.G, ndim, RR, -1, b.V);
        hipLaunchKernelGGL(quadratic_form, dim3(1), dim3(256), 0, st, b.V, lambda, R, b.scalars + 2);
        double h[3];
        int flag = 0;
        if (hipMemcpyAsync(h, b.scalars, 3 * sizeof(double), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipMemcpyAsync(&flag, b.flag, sizeof(int), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            return MTTKRP_ERR_DEVICE;
        if (flag)
            return MTTKRP_ERR_NUMERICAL;   // a Gram Hadamard product was not positive definite
        const double normX = sqrt(h[0]);
        double resid2 = h[0] + h[2] - 2.0 * h[1];
        if (resid2 < 0.0)
            resid2 = 0.0;
        const double fit = normX > 0.0 ? 1.0 - sqrt(resid2) / normX : 1.0;
        if (fits)
            fits[sweep] = fit;
        *iters = sweep + 1;
        if (sweep > 0 && fabs(fit - fit_prev) < tol)
            break;
        fit_prev = fit;
    }
    return hipGetLastError() == hipSuccess ? MTTKRP_OK : MTTKRP_ERR_DEVICE;
}

}  // extern "C"
