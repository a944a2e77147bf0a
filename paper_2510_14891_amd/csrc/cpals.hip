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

constexpr int kSmallRank = 64;     // up to here the R x R matrices are handled in one workgroup's LDS
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


// ---------------------------------------------------------------------------
// Ranks above 64: the R x R matrices no longer fit the LDS of one workgroup.  Gram matrices,
// the Cholesky factorisation and the two triangular solves run blocked from global memory,
// 32 columns at a time, every sum still in a fixed order.
// ---------------------------------------------------------------------------
constexpr int kNB = 32;

// G = A^T A: a 16 x 16 tile of G per workgroup, the rows of A in chunks of 16 through LDS, summed
// in row order.  G(p, q) and G(q, p) add the same products in the same order: G is symmetric bit for bit.
__global__ void __launch_bounds__(256) gram_tiled(const double* __restrict__ A, int64_t I, int R, double* G)
{
    __shared__ double ta[16][17], tb[16][17];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int p0 = blockIdx.y * 16, q0 = blockIdx.x * 16;
    double s = 0.0;
    for (int64_t i0 = 0; i0 < I; i0 += 16) {
        const int64_t i = i0 + ty;
        ta[ty][tx] = i < I && p0 + tx < R ? A[i * R + p0 + tx] : 0.0;
        tb[ty][tx] = i < I && q0 + tx < R ? A[i * R + q0 + tx] : 0.0;
        __syncthreads();
        const int rows = (int)(I - i0 < 16 ? I - i0 : 16);
        for (int r = 0; r < rows; ++r)
            s += ta[r][ty] * tb[r][tx];
        __syncthreads();
    }
    if (p0 + ty < R && q0 + tx < R)
        G[(int64_t)(p0 + ty) * R + q0 + tx] = s;
}

// Diagonal block [j0, j0 + nb) of the blocked factorisation: Cholesky factor of the block in
// LDS by one workgroup, lower triangle written back, the block's upper triangle zeroed.
__global__ void __launch_bounds__(256) chol_diag(double* V, int R, int j0, int nb, int* flag)
{
    __shared__ double B[kNB][kNB + 1];
    if (flag[0])
        return;
    for (int t = threadIdx.x; t < nb * nb; t += 256)
        B[t / nb][t % nb] = V[(int64_t)(j0 + t / nb) * R + j0 + t % nb];
    __syncthreads();
    for (int j = 0; j < nb; ++j) {
        const double piv = B[j][j];
        if (!(piv > 0.0)) {
            if (threadIdx.x == 0)
                flag[0] = 1;
            return;   // uniform: every thread sees the same pivot
        }
        const double dj = sqrt(piv);
        __syncthreads();
        for (int i = j + threadIdx.x; i < nb; i += 256)
            B[i][j] = i == j ? dj : B[i][j] / dj;
        __syncthreads();
        const int n = nb - j - 1;
        for (int t = threadIdx.x; t < n * n; t += 256) {
            const int i = j + 1 + t / n, c = j + 1 + t % n;
            if (c <= i)
                B[i][c] -= B[i][j] * B[c][j];
        }
        __syncthreads();
    }
    for (int t = threadIdx.x; t < nb * nb; t += 256) {
        const int r = t / nb, c = t % nb;
        V[(int64_t)(j0 + r) * R + j0 + c] = c <= r ? B[r][c] : 0.0;
    }
}

// The nb x nb triangle L11 = V[j0 .., j0 ..] into LDS (all of the workgroup's threads).
__device__ __forceinline__ void load_diag_block(const double* __restrict__ V, int R, int j0, int nb, double (*B)[kNB + 1])
{
    for (int t = threadIdx.x; t < kNB * kNB; t += blockDim.x) {
        const int r = t / kNB, c = t % kNB;
        B[r][c] = r < nb && c < nb ? V[(int64_t)(j0 + r) * R + j0 + c] : (r == c ? 1.0 : 0.0);
    }
    __syncthreads();
}

// Rows [r0, r1) of the matrix Y (leading dimension R), columns [j0, j0 + nb): every row is solved
// against L11 (forward: y_c = (y_c - sum_{q < c} L11(c, q) y_q) / L11(c, c), c ascending) or its
// transpose (backward: x_c = (x_c - sum_{q > c} L11(q, c) x_q) / L11(c, c), c descending); one
// thread per row, the row's unknowns in LDS.
constexpr int kSolveThreads = 128;
template <bool FORWARD>
__global__ void __launch_bounds__(kSolveThreads)
solve_diag_rows(const double* __restrict__ L, int R, int j0, int nb, double* Y, int64_t r0, int64_t r1, const int* flag)
{
    __shared__ double B[kNB][kNB + 1];
    __shared__ double ys[kNB][kSolveThreads];
    if (flag[0])
        return;
    load_diag_block(L, R, j0, nb, B);
    const int64_t row = r0 + (int64_t)blockIdx.x * kSolveThreads + threadIdx.x;
    if (row >= r1)
        return;
    const int tid = threadIdx.x;
    for (int c = 0; c < nb; ++c)
        ys[c][tid] = Y[row * R + j0 + c];
    if (FORWARD) {
        for (int c = 0; c < nb; ++c) {
            double v = ys[c][tid];
            for (int q = 0; q < c; ++q)
                v -= B[c][q] * ys[q][tid];
            ys[c][tid] = v / B[c][c];
        }
    } else {
        for (int c = nb - 1; c >= 0; --c) {
            double v = ys[c][tid];
            for (int q = nb - 1; q > c; --q)
                v -= B[q][c] * ys[q][tid];
            ys[c][tid] = v / B[c][c];
        }
    }
    for (int c = 0; c < nb; ++c)
        Y[row * R + j0 + c] = ys[c][tid];
}

// Y(row, c) -= sum_{q < nb} S(row, q) * W(c, q) for rows [r0, r1) and columns [c0, c1), a 16 x 16
// tile per workgroup.  S(row, q) = Y(row, j0 + q); W(c, q) = L(c, j0 + q) (TRANS = false: the
// columns below a block of the forward solve and of the factorisation's trailing update) or
// L(j0 + q, c) (TRANS = true: the columns before a block of the backward solve).  LOWER: only
// entries with c <= row are touched (the factorisation keeps the lower triangle).
template <bool TRANS, bool LOWER>
__global__ void __launch_bounds__(256)
update_tile(const double* __restrict__ L, int R, int j0, int nb, double* Y, int64_t r0, int64_t r1, int c0, int c1,
            const int* flag)
{
    __shared__ double S[16][kNB + 1], W[16][kNB + 1];
    if (flag[0])
        return;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t rt = r0 + (int64_t)blockIdx.y * 16;
    const int ct = c0 + blockIdx.x * 16;
    if (LOWER && ct > rt + 15)
        return;      // a tile above the diagonal
    for (int t = threadIdx.x; t < 16 * kNB; t += 256) {
        const int a = t / kNB, q = t % kNB;
        S[a][q] = q < nb && rt + a < r1 ? Y[(rt + a) * R + j0 + q] : 0.0;
        double w = 0.0;
        if (q < nb && ct + a < c1)
            w = TRANS ? L[(int64_t)(j0 + q) * R + ct + a] : L[(int64_t)(ct + a) * R + j0 + q];
        W[a][q] = w;
    }
    __syncthreads();
    const int64_t row = rt + ty;
    const int c = ct + tx;
    if (row >= r1 || c >= c1 || (LOWER && c > row))
        return;
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < kNB; ++q)
        s += S[ty][q] * W[tx][q];
    Y[row * R + c] -= s;
}

// dst = src (n values) unless the factorisation failed.
__global__ void __launch_bounds__(256) copy_unless_flag(const double* __restrict__ src, double* dst, int64_t n, const int* flag)
{
    if (flag[0])
        return;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e < n)
        dst[e] = src[e];
}

// V := its Cholesky factor (lower triangle; the strict upper triangle keeps stale values that
// nothing reads), block column by block column: factor the diagonal block, solve the panel below
// it (rows of V against L11), update the trailing lower triangle.
void cholesky_blocked(double* V, int R, int* flag, hipStream_t st)
{
    for (int j0 = 0; j0 < R; j0 += kNB) {
        const int nb = R - j0 < kNB ? R - j0 : kNB;
        hipLaunchKernelGGL(chol_diag, dim3(1), dim3(256), 0, st, V, R, j0, nb, flag);
        const int j1 = j0 + nb;
        if (j1 >= R)
            break;
        const int below = R - j1;
        hipLaunchKernelGGL((solve_diag_rows<true>), dim3((unsigned)ceil_div(below, kSolveThreads)), dim3(kSolveThreads), 0, st,
                           (const double*)V, R, j0, nb, V, (int64_t)j1, (int64_t)R, (const int*)flag);
        const unsigned nt = (unsigned)ceil_div(below, 16);
        hipLaunchKernelGGL((update_tile<false, true>), dim3(nt, nt), dim3(256), 0, st,
                           (const double*)V, R, j0, nb, V, (int64_t)j1, (int64_t)R, j1, R, (const int*)flag);
    }
}

// Rows of Y (I x R, in place) := Y V^{-1} with V = L L^T: forward against L block by block, then
// backward against L^T.
void solve_blocked(const double* L, int R, double* Y, int64_t I, const int* flag, hipStream_t st)
{
    const unsigned rb = (unsigned)ceil_div(I, kSolveThreads), rt = (unsigned)ceil_div(I, 16);
    for (int j0 = 0; j0 < R; j0 += kNB) {
        const int nb = R - j0 < kNB ? R - j0 : kNB;
        hipLaunchKernelGGL((solve_diag_rows<true>), dim3(rb), dim3(kSolveThreads), 0, st, L, R, j0, nb, Y, (int64_t)0, I, flag);
        const int j1 = j0 + nb;
        if (j1 < R)
            hipLaunchKernelGGL((update_tile<false, false>), dim3((unsigned)ceil_div(R - j1, 16), rt), dim3(256), 0, st,
                               L, R, j0, nb, Y, (int64_t)0, I, j1, R, flag);
    }
    for (int j0 = (R - 1) / kNB * kNB; j0 >= 0; j0 -= kNB) {
        const int nb = R - j0 < kNB ? R - j0 : kNB;
        hipLaunchKernelGGL((solve_diag_rows<false>), dim3(rb), dim3(kSolveThreads), 0, st, L, R, j0, nb, Y, (int64_t)0, I, flag);
        if (j0 > 0)
            hipLaunchKernelGGL((update_tile<true, false>), dim3((unsigned)ceil_div(j0, 16), rt), dim3(256), 0, st,
                               L, R, j0, nb, Y, (int64_t)0, I, 0, j0, flag);
    }
}

struct Buffers {
    double* M = nullptr;        // max_n I_n x R
    double* G = nullptr;        // d x R x R Gram matrices
    double* V = nullptr;        // R x R
    double* gram_ws = nullptr;  // chunks x R x R
    double* partial = nullptr;  // kNormBlocks + R values
    double* scalars = nullptr;  // ||X||^2, <X, X^>, ||X^||^2
    int* flag = nullptr;
    void* shared_ws = nullptr;  // intermediates of the sweeps that share partial contractions
    ~Buffers()
    {
        (void)hipFree(shared_ws);
        (void)hipFree(M); (void)hipFree(G); (void)hipFree(V); (void)hipFree(gram_ws);
        (void)hipFree(partial); (void)hipFree(scalars); (void)hipFree(flag);
    }
};

void gram(const double* A, int64_t I, int R, double* ws, double* G, hipStream_t st)
{
    if (R > kSmallRank) {
        const unsigned nt = (unsigned)ceil_div(R, 16);
        hipLaunchKernelGGL(gram_tiled, dim3(nt, nt), dim3(256), 0, st, A, I, R, G);
        return;
    }
    const int n_chunks = (int)ceil_div(I, kChunkRows);
    hipLaunchKernelGGL(gram_partial, dim3(n_chunks), dim3(256), (size_t)kChunkRows * R * sizeof(double), st, A, I, R, ws);
    hipLaunchKernelGGL(gram_reduce, dim3((unsigned)ceil_div(R * R, 256)), dim3(256), 0, st, ws, n_chunks, R * R, G);
}


// ---------------------------------------------------------------------------
// Sweep that shares partial contractions between the modes (two passes over X).
// ---------------------------------------------------------------------------

// K(r, j) = prod over the modes m of A_m(r_m, j), r decomposed with the lowest mode fastest;
// row-major with leading dimension R.  One thread per entry.
template <typename T> struct ModeSet {
    const T* A[MTTKRP_MAX_NDIM];
    int64_t ld[MTTKRP_MAX_NDIM];
    int32_t dim[MTTKRP_MAX_NDIM];
    int32_t n;
};
template <typename T>
__global__ void __launch_bounds__(256) khatri_rao_rows(const ModeSet<T> p, int64_t n_entries, int R, T* __restrict__ K)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n_entries)
        return;
    int64_t r = e / R;
    const int j = (int)(e - r * R);
    T v = (T)1;
    for (int m = 0; m < p.n; ++m) {
        const int64_t rn = r / p.dim[m];
        v *= p.A[m][(r - rn * p.dim[m]) * p.ld[m] + j];
        r = rn;
    }
    K[e] = v;
}

// One mode's MTTKRP from a partial contraction.  Tp (P x R, row-major, leading dimension R)
// holds, for every multi-index i of the modes in `p` (lowest fastest, P entries) and every
// column j, the sum of Eq. (elem) over the modes that are not in `p`, without the factors of
// the modes in `p`.  Mode t of the set then gets
//     M(i_t, j) = sum over the other indices of Tp(i, j) * prod_{m in p, m != t} A_m(i_m, j).
// A workgroup owns (i_t, a segment of the other indices, TJ columns): thread (tj, to) adds
// the entries o = to, to + TO, ... of its segment in fp64, the TO subtotals are added in
// order, and the segment totals go to part[i_t][segment][R] for sum_segments.
template <typename T, int TJ>
__global__ void __launch_bounds__(256)
partial_mode_kernel(const ModeSet<T> p, const T* __restrict__ Tp, int t, int R, int64_t n_others,
                    int64_t others_per_seg, int n_seg, double* __restrict__ part)
{
    constexpr int TO = 256 / TJ;
    __shared__ double red[TO][TJ + 1];
    const int tj = threadIdx.x % TJ, to = threadIdx.x / TJ;
    const int64_t it = blockIdx.x;
    const int seg = blockIdx.y;
    const int j = blockIdx.z * TJ + tj;
    const int jj = j < R ? j : R - 1;
    const int64_t o_begin = (int64_t)seg * others_per_seg;
    const int64_t o_end = o_begin + others_per_seg < n_others ? o_begin + others_per_seg : n_others;
    double acc = 0.0;
    for (int64_t o = o_begin + to; o < o_end; o += TO) {
        int64_t rem = o, row = 0, stride = 1;
        double w = 1.0;
        for (int m = 0; m < p.n; ++m) {
            if (m == t) {
                row += it * stride;
            } else {
                const int64_t q = rem / p.dim[m];
                const int64_t im = rem - q * p.dim[m];
                rem = q;
                row += im * stride;
                w *= (double)p.A[m][im * p.ld[m] + jj];
            }
            stride *= p.dim[m];
        }
        acc += (double)Tp[row * R + jj] * w;
    }
    red[to][tj] = acc;
    __syncthreads();
    if (to == 0 && j < R) {
        double v = 0.0;
        for (int q = 0; q < TO; ++q)
            v += red[q][tj];
        part[(it * n_seg + seg) * R + j] = v;
    }
}

// M(i, j) = sum over the segments, in order.  One thread per entry.
template <typename T>
__global__ void __launch_bounds__(256)
sum_segments(const double* __restrict__ part, int64_t n_entries, int R, int n_seg, T* __restrict__ M, int64_t ldM)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n_entries)
        return;
    const int64_t i = e / R;
    const int j = (int)(e - i * R);
    double v = 0.0;
    for (int q = 0; q < n_seg; ++q)
        v += part[(i * n_seg + q) * R + j];
    M[i * ldM + j] = (T)v;
}

template <typename T> struct Calls;
template <> struct Calls<double> {
    static int dense(int nd, const int64_t* d, const double* X, const double* const* f, int R, int k, double* M,
                     void* ws, size_t wsb, void* st)
    { return mttkrp_dense_f64_ws(nd, d, X, f, R, k, M, ws, wsb, st); }
    static int leading(int64_t P, int64_t Q, const double* X, const double* K, int R, double* out, void* ws, size_t wsb, void* st)
    { return mttkrp_contract_leading_f64(P, Q, X, K, R, R, out, R, ws, wsb, st); }
};
template <> struct Calls<float> {
    static int dense(int nd, const int64_t* d, const float* X, const float* const* f, int R, int k, float* M,
                     void* ws, size_t wsb, void* st)
    { return mttkrp_dense_f32_ws(nd, d, X, f, R, k, M, ws, wsb, st); }
    static int leading(int64_t P, int64_t Q, const float* X, const float* K, int R, float* out, void* ws, size_t wsb, void* st)
    { return mttkrp_contract_leading_f32(P, Q, X, K, R, R, out, R, ws, wsb, st); }
};

// Where the modes are cut into a leading set (modes 0 .. s-1, P_L entries) and a trailing
// set (modes s .. d-1, P_R entries), and what lies where in the caller's buffer.
struct SharedPlan {
    int s = 0;
    int64_t PL = 1, PR = 1;
    int max_seg = 1;
    size_t off_TR = 0, off_KL = 0, off_TL = 0, off_part = 0, off_lead = 0, lead_bytes = 0, total = 0;
    // the first pass is a first-mode core call on (P_L, I_s, ..., I_{d-1}); its workspace
    int nd_first = 0;
    int64_t dims_first[MTTKRP_MAX_NDIM];
    size_t off_first = 0, first_bytes = 0;
};

size_t align256(size_t n) { return (n + 255) / 256 * 256; }

// segments of the other indices for one mode: enough workgroups to fill the chip
int segments(int64_t I_t, int64_t n_others)
{
    int64_t n = ceil_div(4096, I_t);
    const int64_t most = ceil_div(n_others, 64);
    if (n > most)
        n = most;
    return (int)(n < 1 ? 1 : n);
}

int plan_shared(int ndim, const int64_t* dims, int R, int sbytes, SharedPlan& sp)
{
    if (!dims || ndim < 2 || R < 1 || (sbytes != 4 && sbytes != 8))
        return MTTKRP_ERR_INVALID_ARG;
    if (ndim > MTTKRP_MAX_NDIM)
        return MTTKRP_ERR_UNSUPPORTED;
    int64_t N = 1;
    for (int m = 0; m < ndim; ++m) {
        if (dims[m] < 1)
            return MTTKRP_ERR_INVALID_ARG;
        if (N > ((int64_t)1 << 57) / dims[m])
            return MTTKRP_ERR_INVALID_ARG;
        N *= dims[m];
    }
    // the cut with the smallest intermediates
    int best = 0;
    int64_t best_sum = 0, PL = 1;
    for (int s = 1; s < ndim; ++s) {
        PL *= dims[s - 1];
        const int64_t PR = N / PL;
        if (PL >= ((int64_t)1 << 31) - 64 || PR >= ((int64_t)1 << 31) - 64)
            continue;
        if (best == 0 || PL + PR < best_sum) {
            best = s;
            best_sum = PL + PR;
        }
    }
    if (best == 0)
        return MTTKRP_ERR_UNSUPPORTED;
    sp.s = best;
    sp.PL = 1;
    for (int m = 0; m < best; ++m)
        sp.PL *= dims[m];
    sp.PR = N / sp.PL;
    const size_t row = (size_t)R * (size_t)sbytes;
    size_t off = 0;
    if (sp.s > 1) {
        sp.off_TR = off;  off += align256((size_t)sp.PL * row);
        sp.off_KL = off;  off += align256((size_t)sp.PL * row);
    }
    if (ndim - sp.s > 1) {
        sp.off_TL = off;  off += align256((size_t)sp.PR * row);
    }
    // segment totals of partial_mode_kernel (fp64), the largest over the modes that use it
    size_t part = 0;
    sp.max_seg = 1;
    for (int k = 0; k < ndim; ++k) {
        const bool left = k < sp.s;
        if ((left && sp.s == 1) || (!left && ndim - sp.s == 1))
            continue;
        const int n_seg = segments(dims[k], (left ? sp.PL : sp.PR) / dims[k]);
        const size_t b = (size_t)dims[k] * (size_t)n_seg * (size_t)R * sizeof(double);
        if (b > part)
            part = b;
        if (n_seg > sp.max_seg)
            sp.max_seg = n_seg;
    }
    sp.off_part = off;  off += align256(part);
    const size_t lead = mttkrp_contract_leading_workspace_bytes(sp.PL, sp.PR, R, sbytes);
    if (lead == (size_t)-1)
        return MTTKRP_ERR_UNSUPPORTED;
    sp.lead_bytes = lead;
    sp.off_lead = off;  off += align256(lead);
    sp.nd_first = 1 + ndim - sp.s;
    sp.dims_first[0] = sp.PL;
    for (int m = sp.s; m < ndim; ++m)
        sp.dims_first[1 + m - sp.s] = dims[m];
    const size_t first = mttkrp_dense_workspace_bytes(sp.nd_first, sp.dims_first, R, 0, sbytes);
    if (first == (size_t)-1)
        return MTTKRP_ERR_UNSUPPORTED;
    sp.first_bytes = first;
    sp.off_first = off;  off += align256(first);
    sp.total = off > 0 ? off : 256;
    // the intermediates must stay small beside the tensor: an eighth of it, or 64 MiB
    double limit = 0.125 * (double)N * sbytes;
    if (limit < 64.0 * 1048576.0)
        limit = 64.0 * 1048576.0;
    if ((double)sp.total > limit)
        return MTTKRP_ERR_UNSUPPORTED;
    return MTTKRP_OK;
}

template <typename T>
int mode_from_partial(const T* Tp, int n, const int64_t* dims, const T* const* factors, int t, int R, T* M,
                      double* part, hipStream_t st)
{
    ModeSet<T> ms;
    ms.n = n;
    int64_t P = 1;
    for (int m = 0; m < n; ++m) {
        ms.A[m] = m == t ? nullptr : factors[m];
        ms.ld[m] = R;
        ms.dim[m] = (int32_t)dims[m];
        P *= dims[m];
    }
    const int64_t n_others = P / dims[t];
    const int n_seg = segments(dims[t], n_others);
    const int64_t per_seg = ceil_div(n_others, n_seg);
    if (dims[t] >= ((int64_t)1 << 31) || n_seg > 65535)
        return MTTKRP_ERR_UNSUPPORTED;
    if (R >= 32) {
        const int64_t jt = ceil_div(R, 32);
        if (jt > 65535)
            return MTTKRP_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((partial_mode_kernel<T, 32>), dim3((unsigned)dims[t], (unsigned)n_seg, (unsigned)jt), dim3(256), 0, st,
                           ms, Tp, t, R, n_others, per_seg, n_seg, part);
    } else if (R > 8) {
        hipLaunchKernelGGL((partial_mode_kernel<T, 16>), dim3((unsigned)dims[t], (unsigned)n_seg, (unsigned)ceil_div(R, 16)), dim3(256), 0, st,
                           ms, Tp, t, R, n_others, per_seg, n_seg, part);
    } else {
        hipLaunchKernelGGL((partial_mode_kernel<T, 8>), dim3((unsigned)dims[t], (unsigned)n_seg, 1), dim3(256), 0, st,
                           ms, Tp, t, R, n_others, per_seg, n_seg, part);
    }
    const int64_t n_entries = dims[t] * (int64_t)R;
    hipLaunchKernelGGL((sum_segments<T>), dim3((unsigned)ceil_div(n_entries, 256)), dim3(256), 0, st,
                       part, n_entries, R, n_seg, M, (int64_t)R);
    return hipGetLastError() == hipSuccess ? MTTKRP_OK : MTTKRP_ERR_DEVICE;
}

// The sweep: M_out[k] for k = 0 .. d-1 in this order; after(k) runs right after M_out[k] has
// been enqueued (CP-ALS updates factors[k] there: later modes then read the new factor, as in
// d separate calls).  Two passes over X: one contracts the trailing modes (every leading
// mode's result follows from it), one the leading modes.
template <typename T, typename After>
int shared_sweep(int ndim, const int64_t* dims, const T* X, const T* const* factors, int R, T* const* M_out,
                 void* workspace, size_t workspace_bytes, void* stream, After after)
{
    if (!X || !factors || !M_out)
        return MTTKRP_ERR_INVALID_ARG;
    SharedPlan sp;
    int rc = plan_shared(ndim, dims, R, (int)sizeof(T), sp);
    if (rc != MTTKRP_OK)
        return rc;
    if (!workspace || workspace_bytes < sp.total)
        return MTTKRP_ERR_WORKSPACE;
    for (int m = 0; m < ndim; ++m)
        if (!factors[m] || !M_out[m])
            return MTTKRP_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    char* const ws = (char*)workspace;
    double* const part = (double*)(ws + sp.off_part);
    const int s = sp.s, nr = ndim - s;
    // pass 1: contraction over the trailing modes
    if (s == 1) {
        rc = Calls<T>::dense(ndim, dims, X, factors, R, 0, M_out[0], ws + sp.off_first, sp.first_bytes, stream);
        if (rc != MTTKRP_OK)
            return rc;
        rc = after(0);
        if (rc != MTTKRP_OK)
            return rc;
    } else {
        const T* f2[MTTKRP_MAX_NDIM];
        f2[0] = nullptr;
        for (int m = 0; m < nr; ++m)
            f2[1 + m] = factors[s + m];
        T* const TR = (T*)(ws + sp.off_TR);
        rc = Calls<T>::dense(sp.nd_first, sp.dims_first, X, f2, R, 0, TR, ws + sp.off_first, sp.first_bytes, stream);
        if (rc != MTTKRP_OK)
            return rc;
        for (int k = 0; k < s; ++k) {
            rc = mode_from_partial<T>(TR, s, dims, factors, k, R, M_out[k], part, st);
            if (rc != MTTKRP_OK)
                return rc;
            rc = after(k);
            if (rc != MTTKRP_OK)
                return rc;
        }
    }
    // pass 2: contraction over the leading modes, whose factors are final now
    const T* K = factors[0];
    if (s > 1) {
        ModeSet<T> ms;
        ms.n = s;
        for (int m = 0; m < s; ++m) {
            ms.A[m] = factors[m];
            ms.ld[m] = R;
            ms.dim[m] = (int32_t)dims[m];
        }
        T* const KL = (T*)(ws + sp.off_KL);
        const int64_t n_entries = sp.PL * (int64_t)R;
        hipLaunchKernelGGL((khatri_rao_rows<T>), dim3((unsigned)ceil_div(n_entries, 256)), dim3(256), 0, st,
                           ms, n_entries, R, KL);
        K = KL;
    }
    T* const TL = nr == 1 ? M_out[ndim - 1] : (T*)(ws + sp.off_TL);
    rc = Calls<T>::leading(sp.PL, sp.PR, X, K, R, TL, ws + sp.off_lead, sp.lead_bytes, stream);
    if (rc != MTTKRP_OK)
        return rc;
    if (nr == 1)
        return after(ndim - 1);
    for (int k = s; k < ndim; ++k) {
        rc = mode_from_partial<T>(TL, nr, dims + s, factors + s, k - s, R, M_out[k], part, st);
        if (rc != MTTKRP_OK)
            return rc;
        rc = after(k);
        if (rc != MTTKRP_OK)
            return rc;
    }
    return MTTKRP_OK;
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

size_t mttkrp_dense_all_modes_shared_bytes(int ndim, const int64_t* dims, int R, int dtype_bytes)
{
    SharedPlan sp;
    if (plan_shared(ndim, dims, R, dtype_bytes, sp) != MTTKRP_OK)
        return 0;
    return sp.total;
}

int mttkrp_dense_all_modes_shared_f64(int ndim, const int64_t* dims, const double* X, const double* const* factors,
                                      int R, double* const* M_out, void* workspace, size_t workspace_bytes,
                                      void* stream)
{
    return shared_sweep<double>(ndim, dims, X, factors, R, M_out, workspace, workspace_bytes, stream,
                                [](int) { return (int)MTTKRP_OK; });
}

int mttkrp_dense_all_modes_shared_f32(int ndim, const int64_t* dims, const float* X, const float* const* factors,
                                      int R, float* const* M_out, void* workspace, size_t workspace_bytes,
                                      void* stream)
{
    return shared_sweep<float>(ndim, dims, X, factors, R, M_out, workspace, workspace_bytes, stream,
                               [](int) { return (int)MTTKRP_OK; });
}

}  // extern "C"

namespace {

int cpals_run(int ndim, const int64_t* dims, const double* X, double* const* factors, double* lambda,
              int R, int max_iters, double tol, int* iters, double* fits, void* stream, bool shared)
{
    if (!dims || !X || !factors || !lambda || !iters || ndim < 2 || R < 1 || max_iters < 1 || !(tol >= 0.0))
        return MTTKRP_ERR_INVALID_ARG;
    if (ndim > MTTKRP_MAX_NDIM || R > MTTKRP_CPALS_MAX_RANK)
        return MTTKRP_ERR_UNSUPPORTED;
    const bool big = R > kSmallRank;
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
    if (big && max_I > (int64_t)65535 * 16)
        return MTTKRP_ERR_UNSUPPORTED;     // the blocked solves' grids
    *iters = 0;
    hipStream_t st = (hipStream_t)stream;
    const int RR = R * R;
    Buffers b;
    // shared sweeps: the intermediates' buffer; without a cut that fits, d separate passes
    SharedPlan sp;
    if (shared && plan_shared(ndim, dims, R, (int)sizeof(double), sp) != MTTKRP_OK)
        shared = false;
    if (shared && hipMalloc(&b.shared_ws, sp.total) != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    const int64_t max_chunks = big ? 1 : ceil_div(max_I, kChunkRows);
    if (hipMalloc(&b.M, (size_t)max_I * R * sizeof(double)) != hipSuccess ||
        hipMalloc(&b.G, (size_t)ndim * RR * sizeof(double)) != hipSuccess ||
        hipMalloc(&b.V, (size_t)RR * sizeof(double)) != hipSuccess ||
        hipMalloc(&b.gram_ws, (size_t)max_chunks * (big ? 1 : RR) * sizeof(double)) != hipSuccess ||
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
    double* mo[MTTKRP_MAX_NDIM];
    for (int m = 0; m < ndim; ++m) {
        cf[m] = factors[m];
        mo[m] = b.M;
    }
    // the update of factor k from its MTTKRP in b.M
    auto update = [&](int k) {
            hipLaunchKernelGGL(hadamard_grams, dim3((unsigned)ceil_div(RR, 256)), dim3(256), 0, st, b.G, ndim, RR, k, b.V);
            if (big) {
                // the rows of M go to A_k (unless the factorisation failed) and are solved there in
                // place: M itself stays for the fit
                cholesky_blocked(b.V, R, b.flag, st);
                const int64_t n = dims[k] * (int64_t)R;
                hipLaunchKernelGGL(copy_unless_flag, dim3((unsigned)ceil_div(n, 256)), dim3(256), 0, st,
                                   (const double*)b.M, factors[k], n, (const int*)b.flag);
                solve_blocked(b.V, R, factors[k], dims[k], b.flag, st);
            } else {
                hipLaunchKernelGGL(cholesky_lower, dim3(1), dim3(256), (size_t)RR * sizeof(double), st, b.V, R, b.flag);
                hipLaunchKernelGGL(solve_rows, dim3((unsigned)ceil_div(dims[k], 32)), dim3(32),
                                   (size_t)(RR + 32 * (R + 1)) * sizeof(double), st, b.V, b.M, dims[k], R, factors[k], b.flag);
            }
            hipLaunchKernelGGL(normalise_columns, dim3(R), dim3(256), 0, st, factors[k], dims[k], R, lambda, b.flag);
            gram(factors[k], dims[k], R, b.gram_ws, b.G + (int64_t)k * RR, st);
            return (int)MTTKRP_OK;
    };
    double fit_prev = 0.0;
    for (int sweep = 0; sweep < max_iters; ++sweep) {
        if (shared) {
            const int rc = shared_sweep<double>(ndim, dims, X, cf, R, mo, b.shared_ws, sp.total, stream, update);
            if (rc != MTTKRP_OK)
                return rc;
        } else {
            for (int k = 0; k < ndim; ++k) {
                const int rc = mttkrp_dense_f64(ndim, dims, X, cf, R, k, b.M, stream);
                if (rc != MTTKRP_OK)
                    return rc;
                update(k);
            }
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

}  // namespace

extern "C" {

int mttkrp_cpals_f64(int ndim, const int64_t* dims, const double* X, double* const* factors, double* lambda,
                     int R, int max_iters, double tol, int* iters, double* fits, void* stream)
{
    return cpals_run(ndim, dims, X, factors, lambda, R, max_iters, tol, iters, fits, stream, false);
}

int mttkrp_cpals_shared_f64(int ndim, const int64_t* dims, const double* X, double* const* factors, double* lambda,
                            int R, int max_iters, double tol, int* iters, double* fits, void* stream)
{
    return cpals_run(ndim, dims, X, factors, lambda, R, max_iters, tol, iters, fits, stream, true);
}

}  // extern "C"
