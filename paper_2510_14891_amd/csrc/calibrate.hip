// Measured ceilings: a read-only stream and back-to-back MFMAs.  C ABI:
// include/mttkrp_calibrate.h.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "../../include/mttkrp.h"
#include "../../include/mttkrp_calibrate.h"

// Written only if a sum hits a value it cannot take, which keeps the probes' work alive.  It has
// external linkage on purpose: stores to an internal variable that nothing reads would be removed
// together with the loads and MFMAs that feed them.
__device__ double mttkrp_calibrate_sink;

namespace {

typedef double double2_t __attribute__((ext_vector_type(2)));
typedef double double4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

constexpr int kStreamBlocks = 8192;
constexpr int kInFlight = 4;      // 16-byte loads in flight per lane
constexpr int kMfmaBlocksPerCu = 8;
constexpr int kAccTiles = 8;      // independent accumulators per wavefront

__global__ void __launch_bounds__(256) stream_read(const double2_t* __restrict__ x, size_t n16)
{
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    double s = 0.0;
    for (; i + (kInFlight - 1) * stride < n16; i += kInFlight * stride) {
        double2_t v[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u)
            v[u] = __builtin_nontemporal_load(&x[i + u * stride]);
#pragma unroll
        for (int u = 0; u < kInFlight; ++u)
            s += v[u].x + v[u].y;
    }
    for (; i < n16; i += stride) {
        const double2_t v = __builtin_nontemporal_load(&x[i]);
        s += v.x + v.y;
    }
    if (s == 1.2345678e300)
        mttkrp_calibrate_sink = s;
}

__global__ void __launch_bounds__(256) mfma_f64(int iters)
{
    double4_t acc[kAccTiles];
#pragma unroll
    for (int a = 0; a < kAccTiles; ++a)
        acc[a] = (double4_t)(0);
    // operands that differ per lane and are neither 0 nor 1
    const double a0 = 0.37 + 0.001 * (double)threadIdx.x;
    const double b0 = 1.13 - 0.002 * (double)(threadIdx.x & 63) + 1e-9 * (double)blockIdx.x;
    for (int t = 0; t < iters; ++t) {
#pragma unroll
        for (int a = 0; a < kAccTiles; ++a)
            acc[a] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b0, acc[a], 0, 0, 0);
    }
    double s = 0.0;
#pragma unroll
    for (int a = 0; a < kAccTiles; ++a)
        s += acc[a][0] + acc[a][1] + acc[a][2] + acc[a][3];
    if (s == 1.2345678e300)
        mttkrp_calibrate_sink = s;
}

__global__ void __launch_bounds__(256) mfma_f32(int iters)
{
    float4_t acc[kAccTiles];
#pragma unroll
    for (int a = 0; a < kAccTiles; ++a)
        acc[a] = (float4_t)(0);
    const float a0 = 0.37f + 0.001f * (float)threadIdx.x;
    const float b0 = 1.13f - 0.002f * (float)(threadIdx.x & 63) + 1e-6f * (float)(blockIdx.x & 1023);
    for (int t = 0; t < iters; ++t) {
#pragma unroll
        for (int a = 0; a < kAccTiles; ++a)
            acc[a] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0, acc[a], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int a = 0; a < kAccTiles; ++a)
        s += acc[a][0] + acc[a][1] + acc[a][2] + acc[a][3];
    if (s == 1.2345678e30f)
        mttkrp_calibrate_sink = (double)s;
}

// Mean milliseconds of `launches` launches of f on st, after two untimed ones.
template <typename F> int timed(F f, int launches, hipStream_t st, float* ms_mean)
{
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
        if (e0) (void)hipEventDestroy(e0);
        return MTTKRP_ERR_DEVICE;
    }
    f();
    f();
    int rc = MTTKRP_OK;
    float ms = 0.0f;
    if (hipEventRecord(e0, st) != hipSuccess)
        rc = MTTKRP_ERR_DEVICE;
    for (int i = 0; i < launches && rc == MTTKRP_OK; ++i)
        f();
    if (rc == MTTKRP_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                            hipEventElapsedTime(&ms, e0, e1) != hipSuccess || hipGetLastError() != hipSuccess))
        rc = MTTKRP_ERR_DEVICE;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *ms_mean = ms / (float)launches;
    return rc;
}

}  // namespace

extern "C" {

int mttkrp_calibrate_stream(const void* buf, size_t bytes, int launches, float* ms_mean, void* stream)
{
    if (!buf || !ms_mean || launches < 1 || bytes < 16 || (bytes & 15) || ((uintptr_t)buf & 15))
        return MTTKRP_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > (size_t)kStreamBlocks)
        blocks = kStreamBlocks;
    return timed([&] { hipLaunchKernelGGL(stream_read, dim3((unsigned)blocks), dim3(256), 0, st,
                                          (const double2_t*)buf, n16); },
                 launches, st, ms_mean);
}

int mttkrp_calibrate_mfma(int dtype_bytes, double gflop_per_launch, int launches, float* ms_mean, double* flop,
                          void* stream)
{
    if (!ms_mean || !flop || launches < 1 || (dtype_bytes != 4 && dtype_bytes != 8) ||
        !(gflop_per_launch > 0.0) || gflop_per_launch > 1e6)
        return MTTKRP_ERR_INVALID_ARG;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return MTTKRP_ERR_DEVICE;
    hipStream_t st = (hipStream_t)stream;
    const int blocks = cus * kMfmaBlocksPerCu;
    const double flop_per_iter = (double)blocks * 4.0 * kAccTiles * 2048.0;   // 4 wavefronts per workgroup
    double it = gflop_per_launch * 1e9 / flop_per_iter;
    int iters = (int)it;
    if ((double)iters < it)
        iters += 1;
    if (iters < 1)
        iters = 1;
    *flop = flop_per_iter * iters;
    if (dtype_bytes == 8)
        return timed([&] { hipLaunchKernelGGL(mfma_f64, dim3(blocks), dim3(256), 0, st, iters); }, launches, st, ms_mean);
    return timed([&] { hipLaunchKernelGGL(mfma_f32, dim3(blocks), dim3(256), 0, st, iters); }, launches, st, ms_mean);
}

}  // extern "C"
