// The paper's three matrix-free schedules (Sec. III-B ELEM, III-C SUB, III-D
// TILE) as plain HIP kernels, written from the text's description of what each
// schedule does, and the tile-volume heuristic of Sec. IV-C, Eq. (heuristic).
// They exist for side-by-side measurements against the streaming kernel: what
// is kept is what defines each schedule (who owns which entries, how indices
// are formed, how often X and the factors are read, where atomics are used),
// not any tuning.  C ABI and conventions: include/mttkrp_ablation.h.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "../../include/mttkrp.h"
#include "../../include/mttkrp_ablation.h"

namespace {

constexpr int kTeamThreads = 128;   // workgroup size: b_x * b_y = 128 (Sec. IV-A)

template <typename T> struct AblArgs {
    const T* X;
    const T* A[MTTKRP_MAX_NDIM];
    T* M;
    int64_t dims[MTTKRP_MAX_NDIM];
    int64_t strides[MTTKRP_MAX_NDIM];
    int64_t tiles[MTTKRP_MAX_NDIM];   // tiles along each mode (1 for mode k)
    int64_t tiles_per_sub;
    int64_t width;
    int64_t n_units;                  // tensor entries (ELEM) or tiles (SUB, TILE)
    int32_t ndim, R, k;
    int32_t by;                       // lanes of one team thread (split the R columns)
    int32_t atomic;                   // 0: conflict-free plain store (SUB)
};

template <typename T> __device__ __forceinline__ void atomic_add(T* p, T v)
{
    unsafeAtomicAdd(p, v);   // hardware floating-point atomic add
}

template <typename T> __global__ void __launch_bounds__(256) fill_zero(T* p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n)
        p[i] = (T)0;
}

// Sec. III-B: entry i of X belongs to team thread i.  Its multi-index comes from
// divisions of the linear index; for each of its columns j the lane forms
// y * prod_{m != k} A_m(i_m, j) and adds it to M(i_k, j) atomically.
template <typename T> __global__ void __launch_bounds__(kTeamThreads) elem_kernel(const AblArgs<T> p)
{
    const int bx = kTeamThreads / p.by;
    const int px = (int)threadIdx.x / p.by;
    const int py = (int)threadIdx.x - px * p.by;
    // a launch holds at most 2^32 threads, so team threads stride over the entries
    for (int64_t i = (int64_t)blockIdx.x * bx + px; i < p.n_units; i += (int64_t)gridDim.x * bx) {
        const T y = p.X[i];
        int64_t idx[MTTKRP_MAX_NDIM];
        int64_t rem = i;
#pragma unroll
        for (int m = 0; m < MTTKRP_MAX_NDIM; ++m) {
            idx[m] = 0;
            if (m < p.ndim) {
                const int64_t q = rem / p.dims[m];
                idx[m] = rem - q * p.dims[m];
                rem = q;
            }
        }
        int64_t ik = 0;
#pragma unroll
        for (int m = 0; m < MTTKRP_MAX_NDIM; ++m)
            if (m == p.k)
                ik = idx[m];
        for (int j = py; j < p.R; j += p.by) {
            T phi = y;
#pragma unroll
            for (int m = 0; m < MTTKRP_MAX_NDIM; ++m)
                if (m < p.ndim && m != p.k)
                    phi *= p.A[m][idx[m] * p.R + j];
            atomic_add(&p.M[ik * p.R + j], phi);
        }
    }
}

// Sec. III-C / III-D: team thread u owns tile t of subtensor n.  The tile is the
// cube [a_m, a_m + len_m) in every mode m != k (anchor a, clipped at the edges).
// For each of its columns the lane walks the tile with an odometer (additions
// only), re-reading X, multiplying the d-1 factor entries and summing; the tile's
// sum goes to M(n, j) by one atomic add (TILE) or one plain store (SUB, where the
// tile is the whole subtensor and nobody else writes row n).
template <typename T> __global__ void __launch_bounds__(kTeamThreads) tile_kernel(const AblArgs<T> p)
{
    const int bx = kTeamThreads / p.by;
    const int px = (int)threadIdx.x / p.by;
    const int py = (int)threadIdx.x - px * p.by;
    // a launch holds at most 2^32 threads, so team threads stride over the tiles
    for (int64_t u = (int64_t)blockIdx.x * bx + px; u < p.n_units; u += (int64_t)gridDim.x * bx) {
        const int64_t n = u / p.tiles_per_sub;
        int64_t t = u - n * p.tiles_per_sub;
        int64_t a[MTTKRP_MAX_NDIM], len[MTTKRP_MAX_NDIM];
        int64_t base = 0, vol = 1;
#pragma unroll
        for (int m = 0; m < MTTKRP_MAX_NDIM; ++m) {
            a[m] = 0;
            len[m] = 1;
            if (m < p.ndim) {
                if (m == p.k) {
                    base += n * p.strides[m];
                } else {
                    const int64_t q = t / p.tiles[m];
                    const int64_t tc = t - q * p.tiles[m];
                    t = q;
                    a[m] = tc * p.width;
                    len[m] = p.dims[m] - a[m] < p.width ? p.dims[m] - a[m] : p.width;
                    base += a[m] * p.strides[m];
                    vol *= len[m];
                }
            }
        }
        for (int j = py; j < p.R; j += p.by) {
            int64_t loc[MTTKRP_MAX_NDIM];
#pragma unroll
            for (int m = 0; m < MTTKRP_MAX_NDIM; ++m)
                loc[m] = 0;
            int64_t off = 0;
            T pi = (T)0;
            for (int64_t e = 0; e < vol; ++e) {
                T phi = p.X[base + off];
#pragma unroll
                for (int m = 0; m < MTTKRP_MAX_NDIM; ++m)
                    if (m < p.ndim && m != p.k)
                        phi *= p.A[m][(a[m] + loc[m]) * p.R + j];
                pi += phi;
                bool carry = true;
#pragma unroll
                for (int m = 0; m < MTTKRP_MAX_NDIM; ++m) {
                    if (m < p.ndim && m != p.k && carry) {
                        loc[m] += 1;
                        off += p.strides[m];
                        if (loc[m] < len[m]) {
                            carry = false;
                        } else {
                            off -= loc[m] * p.strides[m];
                            loc[m] = 0;
                        }
                    }
                }
            }
            if (p.atomic)
                atomic_add(&p.M[n * p.R + j], pi);
            else
                p.M[n * p.R + j] = pi;
        }
    }
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

template <typename T>
int run(int schedule, int ndim, const int64_t* dims, const T* X, const T* const* factors, int R, int k,
        int64_t tile_width, T* M, void* stream)
{
    if (!dims || !X || !factors || !M || ndim < 2 || R < 1 || k < 0 || k >= ndim)
        return MTTKRP_ERR_INVALID_ARG;
    if (ndim > MTTKRP_MAX_NDIM)
        return MTTKRP_ERR_UNSUPPORTED;
    if (schedule != MTTKRP_SCHEDULE_ELEM && schedule != MTTKRP_SCHEDULE_SUB && schedule != MTTKRP_SCHEDULE_TILE)
        return MTTKRP_ERR_INVALID_ARG;
    if (schedule == MTTKRP_SCHEDULE_TILE && tile_width < 1)
        return MTTKRP_ERR_INVALID_ARG;
    AblArgs<T> a{};
    int64_t N = 1;
    for (int m = 0; m < ndim; ++m) {
        if (dims[m] < 1)
            return MTTKRP_ERR_INVALID_ARG;
        if (m != k && !factors[m])
            return MTTKRP_ERR_INVALID_ARG;
        if (dims[m] >= ((int64_t)1 << 31))
            return MTTKRP_ERR_UNSUPPORTED;
        if (N > (((int64_t)1 << 60) / (int64_t)sizeof(T)) / dims[m])
            return MTTKRP_ERR_INVALID_ARG;
        a.dims[m] = dims[m];
        a.strides[m] = N;
        a.A[m] = m == k ? nullptr : factors[m];
        N *= dims[m];
    }
    a.X = X;
    a.M = M;
    a.ndim = ndim;
    a.R = R;
    a.k = k;
    int by = 1;
    while (by < R && by < 64)
        by *= 2;
    a.by = by;
    const int bx = kTeamThreads / by;
    hipStream_t st = (hipStream_t)stream;

    if (schedule == MTTKRP_SCHEDULE_ELEM) {
        a.n_units = N;
        a.atomic = 1;
    } else {
        const bool sub = schedule == MTTKRP_SCHEDULE_SUB;
        a.width = sub ? ((int64_t)1 << 31) : tile_width;     // SUB: one tile spans every extent
        a.tiles_per_sub = 1;
        for (int m = 0; m < ndim; ++m) {
            a.tiles[m] = m == k ? 1 : ceil_div(dims[m], a.width);
            if (a.tiles_per_sub > (((int64_t)1 << 40)) / a.tiles[m])
                return MTTKRP_ERR_UNSUPPORTED;
            a.tiles_per_sub *= a.tiles[m];
        }
        a.n_units = a.tiles_per_sub * dims[k];
        a.atomic = sub ? 0 : 1;
    }
    int64_t blocks = ceil_div(a.n_units, bx);
    if (blocks > ((int64_t)1 << 24))      // 2^24 workgroups of 128 threads; the kernels stride beyond that
        blocks = (int64_t)1 << 24;

    if (a.atomic) {
        const int64_t n_out = dims[k] * (int64_t)R;
        hipLaunchKernelGGL(fill_zero<T>, dim3((unsigned)ceil_div(n_out, 256)), dim3(256), 0, st, M, n_out);
    }
    if (schedule == MTTKRP_SCHEDULE_ELEM)
        hipLaunchKernelGGL(elem_kernel<T>, dim3((unsigned)blocks), dim3(kTeamThreads), 0, st, a);
    else
        hipLaunchKernelGGL(tile_kernel<T>, dim3((unsigned)blocks), dim3(kTeamThreads), 0, st, a);
    return hipGetLastError() == hipSuccess ? MTTKRP_OK : MTTKRP_ERR_DEVICE;
}

}  // namespace

extern "C" {

int mttkrp_ablation_f64(int schedule, int ndim, const int64_t* dims, const double* X,
                        const double* const* factors, int R, int k, int64_t tile_width, double* M,
                        void* stream)
{
    return run<double>(schedule, ndim, dims, X, factors, R, k, tile_width, M, stream);
}

int mttkrp_ablation_f32(int schedule, int ndim, const int64_t* dims, const float* X,
                        const float* const* factors, int R, int k, int64_t tile_width, float* M,
                        void* stream)
{
    return run<float>(schedule, ndim, dims, X, factors, R, k, tile_width, M, stream);
}

int mttkrp_tile_volume(int ndim, const int64_t* dims, int64_t cache_bytes, int value_bytes,
                       int64_t tiles_per_unit, int64_t* width, int64_t* volume)
{
    if (!dims || !width || !volume || ndim < 2 || ndim > MTTKRP_MAX_NDIM || cache_bytes < 1 ||
        value_bytes < 1 || tiles_per_unit < 1 || cache_bytes > ((int64_t)1 << 40) ||
        tiles_per_unit > ((int64_t)1 << 20) || value_bytes > 64)
        return MTTKRP_ERR_INVALID_ARG;
    int64_t cap = dims[0];
    for (int m = 0; m < ndim; ++m) {
        if (dims[m] < 1)
            return MTTKRP_ERR_INVALID_ARG;
        if (dims[m] < cap)
            cap = dims[m];
    }
    // largest w with w^(d-1) <= (s_LM / 4) / (s_f * c / 2), i.e. w^(d-1) * 2 * s_f * c <= s_LM
    const int64_t unit = 2 * (int64_t)value_bytes * tiles_per_unit;
    auto fits = [&](int64_t w) {
        int64_t v = unit;
        for (int e = 0; e < ndim - 1; ++e) {
            if (v > cache_bytes / w)
                return false;
            v *= w;
        }
        return v <= cache_bytes;
    };
    int64_t w = 1;
    while (w < cap && fits(w + 1))
        w += 1;
    int64_t v = 1;
    for (int e = 0; e < ndim - 1; ++e)
        v *= w;
    *width = w;
    *volume = v;
    return MTTKRP_OK;
}

}  // extern "C"
