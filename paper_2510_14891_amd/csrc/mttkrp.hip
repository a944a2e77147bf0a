// Matrix-free dense mode-k MTTKRP for gfx950 (MI355X): kernels and C ABI.
//
// Computes M(n,j) = sum_{i: i_k=n} X(i) prod_{m!=k} A_m(i_m,j)  (paper Sec. II-B,
// Eq. (elem), lambda = 1) in one streaming pass over X.
//
// How the sum is organised (our own schedule; the paper's ELEM/SUB/TILE
// schedules of Sec. III recompute the whole product per element):
//
//   rows    = mode 0 (contiguous in memory, so loads along it coalesce)
//   batch   = mode k when k != 0 (one output row per batch value)
//   columns = every other mode; the lowest suitable one is the "inner" mode,
//             the rest are "outer" modes walked by a wave-uniform odometer
//
//   T(r, j)  = sum_c X(r, c) * P_c(j),   P_c(j) = prod_{column modes} A_m(c_m, j)
//   k == 0:  M(r, j) = T(r, j)
//   k != 0:  M(i_k, j) = sum_r A_0(r, j) * T(r, j)        (epilogue, once per item)
//
// The first line is a dense (rows x columns) * (columns x R) contraction with
// the right operand generated on the fly: a wavefront owns 16*RB rows, walks
// its columns four at a time and issues RB*JB 16x16x4 MFMAs per step, the A
// operand being X exactly as it lies in memory and the B operand being four
// freshly built partial Khatri-Rao rows.  Wavefronts never synchronise; each
// one writes a partial tile which a small second kernel sums in a fixed order
// (deterministic, no atomics; Sec. III-D's atomics are what this replaces).
#include <hip/hip_runtime.h>

#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <new>

#include "../../include/mttkrp.h"

namespace {

constexpr int kMaxOuter = MTTKRP_MAX_NDIM - 2;
constexpr int kWaves = 4;           // independent wavefronts per workgroup
constexpr int kBlockThreads = 64 * kWaves;
constexpr int kMaxDevices = 16;

typedef double double4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// 16x16x4 MFMA of each data type.  Operand A: lane l holds A[l%16][l/16];
// operand B: lane l holds B[l/16][l%16]; result: lane l, register q holds
// D[row(l,q)][l%16].
template <typename T> struct Mfma;
template <> struct Mfma<double> {
    typedef double4_t acc_t;
    static __device__ __forceinline__ acc_t run(double a, double b, acc_t c) {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int lane, int q) { return 4 * q + (lane >> 4); }
};
template <> struct Mfma<float> {
    typedef float4_t acc_t;
    static __device__ __forceinline__ acc_t run(float a, float b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int lane, int q) { return 4 * (lane >> 4) + q; }
};

template <typename T> struct StreamArgs {
    const T* X;
    const T* A_row;              // factor of mode 0; epilogue weight when k != 0
    const T* A_in;               // factor of the inner column mode, null if none
    const T* A_out[kMaxOuter];   // factors of the outer column modes
    T* out;                      // M itself or the partial-sum workspace
    int64_t sx_in;               // stride of the inner mode in X (elements)
    int64_t sx_batch;            // stride of mode k in X (0 when k == 0)
    int64_t sx_out[kMaxOuter];
    int64_t o_total;             // outer iterations in all
    int64_t o_per_item;          // outer iterations per work item
    int32_t dim_out[kMaxOuter];
    int32_t n_out;
    int32_t I0, I_in, R;
    int32_t first_mode;          // 1 when k == 0
    int32_t n_rowblk, n_jchunk, n_batch, n_isplit;
    int32_t cols_per_isplit;     // inner columns per inner split (multiple of 4)
    int32_t n_items;
    int32_t n_slots;             // partial slots per output row (k != 0)
    int32_t xcd_remap;
    int32_t no_inner;            // 1: no column mode at all; A_in is only a readable dummy
};

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uni64(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// One wavefront = one work item = (row block, column-block chunk, batch value,
// inner split, outer split).  No LDS, no barriers.
//
// Outer column modes: the first one ("mid") is walked by a plain counter; the
// others ("far") only change when mid wraps, and are then re-derived from the
// linear outer index by division (rare).
template <typename T, int RB, int JB>
__global__ void __launch_bounds__(kBlockThreads, 2)
mttkrp_stream_kernel(const StreamArgs<T> p)
{
    typedef Mfma<T> MF;
    typedef typename MF::acc_t acc_t;

    const int lane = threadIdx.x & 63;
    const int wave = uni((int)(threadIdx.x >> 6));
    uint32_t blk = blockIdx.x;
    if (p.xcd_remap)   // workgroups go round-robin over the 8 XCDs: give each XCD a contiguous range
        blk = (blk & 7u) * (gridDim.x >> 3) + (blk >> 3);
    uint32_t it = blk * kWaves + wave;
    if (it >= (uint32_t)p.n_items)
        return;
    const int rowblk = uni((int)(it % (uint32_t)p.n_rowblk));  it /= (uint32_t)p.n_rowblk;
    const int jchunk = uni((int)(it % (uint32_t)p.n_jchunk));  it /= (uint32_t)p.n_jchunk;
    const int batch = uni((int)(it % (uint32_t)p.n_batch));    it /= (uint32_t)p.n_batch;
    const int isp = uni((int)(it % (uint32_t)p.n_isplit));     it /= (uint32_t)p.n_isplit;
    const int osp = uni((int)it);

    const int il = lane & 15;   // row inside a 16-row block (operand A) = column inside a 16-column block (B, D)
    const int kk = lane >> 4;   // which of the step's four columns this lane feeds
    const int R = p.R;

    // Rows: the last row block is shifted down to end at I0 so that every load
    // stays inside the tensor; rows it shares with the previous block are
    // dropped in the epilogue.  With fewer than 16 rows lanes clamp instead.
    const int first_row = rowblk * (16 * RB);
    int row_base = first_row;
    if (row_base + 16 * RB > p.I0)
        row_base = p.I0 > 16 * RB ? p.I0 - 16 * RB : 0;
    const int il_c = min(il, p.I0 - 1 - row_base);

    // Columns of the output (j): clamp for loads, mask at the stores.
    const int j_first = jchunk * (16 * JB);
    int jc[JB];
#pragma unroll
    for (int jb = 0; jb < JB; ++jb)
        jc[jb] = min(j_first + 16 * jb + il, R - 1);

    // Range of this item in the (outer iteration, inner column) space.
    const int ia_begin = isp * p.cols_per_isplit;
    const int ia_end = min(p.I_in, ia_begin + p.cols_per_isplit);
    const int steps_in = (ia_end - ia_begin + 3) >> 2;
    const int64_t o_begin = (int64_t)osp * p.o_per_item;
    const int o_count = uni((int)min(p.o_per_item, p.o_total - o_begin));

    const T* const xlane = p.X + (int64_t)batch * p.sx_batch + (row_base + il_c);
    const int64_t x_step = 4 * p.sx_in;
    const bool no_inner = p.no_inner != 0;   // then A_in is a readable dummy and b = 1
    const int dim_mid = p.dim_out[0];        // 1 when there is no outer mode
    const int64_t sx_mid = p.sx_out[0];
    const T* const A_mid = p.n_out > 0 ? p.A_out[0] : p.A_in;   // dummy when unused
    const bool has_mid = p.n_out > 0;

    // State of the outer walk (all wave-uniform except the factor values).
    int i_mid = 0;
    int i_far[kMaxOuter];         // i_far[m] for outer modes m >= 1
    int64_t xoff_far = 0;         // X offset of the far modes
    T Qfar[JB];                   // product of the far modes' factor entries
    T Q[JB];                      // ... times the mid mode's entry: weight of the sweep being issued
    T mid_next[JB];               // mid factor entries of row i_mid + 1, loaded one sweep ahead
    auto load_mid = [&](int i, T (&dst)[JB]) {
        const T* a = A_mid + (int64_t)(has_mid ? i : 0) * R;
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            dst[jb] = a[jc[jb]];
    };
    auto load_far = [&]() {       // Qfar and Q from the current indices (rare; waits for its loads)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            Qfar[jb] = (T)1;
#pragma unroll
        for (int m = 1; m < kMaxOuter; ++m) {
            if (m < p.n_out) {
                const T* a = p.A_out[m] + (int64_t)i_far[m] * R;
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
                    Qfar[jb] *= a[jc[jb]];
            }
        }
        T mid_now[JB];
        load_mid(i_mid, mid_now);
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            Q[jb] = has_mid ? Qfar[jb] * mid_now[jb] : Qfar[jb];
    };
    {   // decode the first outer index of this item (the only divisions of the walk)
        int64_t t = uni64(o_begin / dim_mid);
        i_mid = uni((int)(o_begin - t * dim_mid));
#pragma unroll
        for (int m = 1; m < kMaxOuter; ++m) {
            i_far[m] = 0;
            if (m < p.n_out) {
                const int64_t tn = uni64(t / p.dim_out[m]);
                i_far[m] = uni((int)(t - tn * p.dim_out[m]));
                t = tn;
                xoff_far += (int64_t)i_far[m] * p.sx_out[m];
            }
        }
    }
    load_far();
    load_mid(min(i_mid + 1, dim_mid - 1), mid_next);

    int ia = ia_begin;
    int s_in = 0;
    const T* xp = xlane + xoff_far + (int64_t)i_mid * sx_mid + (int64_t)(ia_begin + kk) * p.sx_in;

    // Issue the loads of the step the cursor points at into one operand set.
    auto issue = [&](T (&xn)[RB], T (&bn)[JB], T (&qn)[JB]) {
        // lanes whose column lies beyond the inner range read a valid column instead and get q = 0
        const int over = max(ia + kk - (ia_end - 1), 0);
        const T* xe = xp - (int64_t)over * p.sx_in;
        const int kk_c = kk - over;
#pragma unroll
        for (int r = 0; r < RB; ++r)
            xn[r] = __builtin_nontemporal_load(xe + 16 * r);
        const T* b = p.A_in + (int64_t)(ia + kk_c) * R;
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            bn[jb] = b[jc[jb]];
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            qn[jb] = over == 0 ? Q[jb] : (T)0;
    };
    // Move the cursor one step on (wave-uniform control flow).  Past the last
    // step the cursor parks: it keeps pointing at the last step with weight 0,
    // so that a surplus issue stays in bounds and adds nothing.
    int steps_left = o_count * steps_in - 1;   // steps after the one the cursor points at
    auto advance = [&]() {
        if (steps_left <= 0) {
#pragma unroll
            for (int jb = 0; jb < JB; ++jb)
                Q[jb] = (T)0;
            return;
        }
        steps_left -= 1;
        s_in += 1;
        if (s_in < steps_in) {
            ia += 4;
            xp += x_step;
        } else {                  // next sweep
            s_in = 0;
            ia = ia_begin;
            i_mid += 1;
            if (i_mid >= dim_mid) {   // mid wraps: carry into the far modes
                i_mid = 0;
                bool carry = true;
#pragma unroll
                for (int m = 1; m < kMaxOuter; ++m) {
                    if (m < p.n_out && carry) {
                        i_far[m] += 1;
                        xoff_far += p.sx_out[m];
                        if (i_far[m] < p.dim_out[m]) {
                            carry = false;
                        } else {
                            xoff_far -= (int64_t)i_far[m] * p.sx_out[m];
                            i_far[m] = 0;
                        }
                    }
                }
                load_far();
            } else {
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
                    Q[jb] = Qfar[jb] * mid_next[jb];
            }
            load_mid(min(i_mid + 1, dim_mid - 1), mid_next);
            xp = xlane + xoff_far + (int64_t)i_mid * sx_mid + (int64_t)(ia_begin + kk) * p.sx_in;
        }
    };

    acc_t acc[RB][JB];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            acc[r][jb] = (acc_t)(0);
    auto consume = [&](const T (&xc)[RB], const T (&bn)[JB], const T (&qn)[JB]) {
        T bc[JB];
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            bc[jb] = (no_inner ? (T)1 : bn[jb]) * qn[jb];
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int jb = 0; jb < JB; ++jb)
                acc[r][jb] = MF::run(xc[r], bc[jb], acc[r][jb]);
    };

    // Two operand sets in flight, no register copies: while one step's MFMAs
    // run, the loads of the next step are outstanding.  Steps are taken in
    // pairs; an odd count is padded by one parked (zero-weight) step.
    T x0[RB], b0[JB], q0[JB], x1[RB], b1[JB], q1[JB];
    const int n_pairs = (o_count * steps_in + 1) >> 1;
    issue(x0, b0, q0);
    for (int pr = 0; pr < n_pairs; ++pr) {
        advance();
        issue(x1, b1, q1);
        consume(x0, b0, q0);
        advance();
        issue(x0, b0, q0);
        consume(x1, b1, q1);
    }

    // Epilogue.
    if (p.first_mode) {
        const int64_t split = (int64_t)osp * p.n_isplit + isp;
        T* o = p.out + split * ((int64_t)p.I0 * R);
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = row_base + 16 * r + MF::row(lane, q);
                    const int j = j_first + 16 * jb + il;
                    if (row >= first_row && row < p.I0 && j < R)
                        o[(int64_t)row * R + j] = acc[r][jb][q];
                }
    } else {
        const int64_t slot = ((int64_t)osp * p.n_isplit + isp) * p.n_rowblk + rowblk;
        T* o = p.out + ((int64_t)batch * p.n_slots + slot) * R;
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) {
            double v = 0.0;
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = row_base + 16 * r + MF::row(lane, q);
                    const bool ok = row >= first_row && row < p.I0;
                    const int row_c = min(row, p.I0 - 1);
                    const T w = p.A_row[(int64_t)row_c * R + jc[jb]];
                    v += ok ? (double)acc[r][jb][q] * (double)w : 0.0;
                }
            v += __shfl_xor(v, 16);
            v += __shfl_xor(v, 32);
            const int j = j_first + 16 * jb + il;
            if (kk == 0 && j < R)
                o[j] = (T)v;
        }
    }
}

// M(n, j) = sum over slots of the partial sums, in slot order, in fp64.
template <typename T>
__global__ void __launch_bounds__(256)
mttkrp_combine_kernel(const T* __restrict__ ws, T* __restrict__ M, int64_t n_elems, int R,
                      int n_slots, int64_t stride_row, int64_t stride_slot)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_elems)
        return;
    const int64_t n = e / R;
    const int j = (int)(e - n * R);
    const T* src = ws + n * stride_row + j;
    double s = 0.0;
    int t = 0;
    for (; t + 8 <= n_slots; t += 8) {
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = (double)src[(int64_t)(t + u) * stride_slot];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            s += v[u];
    }
    for (; t < n_slots; ++t)
        s += (double)src[(int64_t)t * stride_slot];
    M[e] = (T)s;
}

// ---------------------------------------------------------------------------
// Host side: plan, launch, C ABI
// ---------------------------------------------------------------------------

struct Tuning {
    int64_t row_blocks = 0;
    int64_t target_items = 0;
    int64_t max_steps = 0;
    int64_t xcd_remap = 0;
    int64_t ws_percent = 0;
};
Tuning g_tune;
std::mutex g_mutex;

struct Plan {
    int ndim = 0, R = 0, k = 0, sbytes = 0;
    int64_t dims[MTTKRP_MAX_NDIM];
    int64_t strides[MTTKRP_MAX_NDIM];
    int64_t N = 0;
    int RB = 1, JB = 1, n_jchunk = 1;
    int inner = -1;
    int n_out = 0;
    int out_modes[kMaxOuter];
    int64_t I_in = 1;
    int n_rowblk = 1, n_batch = 1, n_isplit = 1, cols_per_isplit = 4;
    int64_t o_total = 1, o_per_item = 1, n_osplit = 1;
    int64_t n_items = 0;
    int64_t n_slots = 1;       // partial sums per output entry
    int64_t steps_per_item = 0;
    size_t ws_bytes = 0;
    bool xcd_remap = true;
};

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

int validate(int ndim, const int64_t* dims, int R, int k, int sbytes)
{
    if (!dims || ndim < 2 || R < 1 || k < 0 || k >= ndim || (sbytes != 4 && sbytes != 8))
        return MTTKRP_ERR_INVALID_ARG;
    int64_t n = 1;
    for (int m = 0; m < ndim && m < 64; ++m) {
        if (dims[m] < 1)
            return MTTKRP_ERR_INVALID_ARG;
        if (n > (INT64_MAX / 16) / dims[m])   // N * 8 bytes must fit int64 with headroom
            return MTTKRP_ERR_INVALID_ARG;
        n *= dims[m];
    }
    if (ndim > MTTKRP_MAX_NDIM)
        return MTTKRP_ERR_UNSUPPORTED;
    for (int m = 0; m < ndim; ++m)
        if (dims[m] >= (int64_t)1 << 31)
            return MTTKRP_ERR_UNSUPPORTED;
    if ((int64_t)R >= ((int64_t)1 << 27))
        return MTTKRP_ERR_UNSUPPORTED;
    return MTTKRP_OK;
}

int make_plan(int ndim, const int64_t* dims, int R, int k, int sbytes, Plan& pl)
{
    int rc = validate(ndim, dims, R, k, sbytes);
    if (rc != MTTKRP_OK)
        return rc;
    Tuning tn;
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        tn = g_tune;
    }
    pl.ndim = ndim; pl.R = R; pl.k = k; pl.sbytes = sbytes;
    int64_t s = 1;
    for (int m = 0; m < ndim; ++m) {
        pl.dims[m] = dims[m];
        pl.strides[m] = s;
        s *= dims[m];
    }
    pl.N = s;
    const int64_t I0 = dims[0];

    // Row blocks per wavefront: the largest RB (<= 4) whose padding waste is
    // within 10 % of the best achievable; never more rows than the tensor has.
    {
        int best = 1;
        double best_eff = 0.0;
        const int rb_max = I0 >= 16 ? (int)(I0 / 16 < 4 ? I0 / 16 : 4) : 1;
        double eff[5] = {0, 0, 0, 0, 0};
        for (int rb = 1; rb <= rb_max; ++rb) {
            eff[rb] = (double)I0 / (double)(ceil_div(I0, 16 * rb) * 16 * rb);
            if (eff[rb] > best_eff)
                best_eff = eff[rb];
        }
        for (int rb = rb_max; rb >= 1; --rb)
            if (eff[rb] >= 0.9 * best_eff) { best = rb; break; }
        if (tn.row_blocks >= 1 && tn.row_blocks <= rb_max)
            best = (int)tn.row_blocks;
        pl.RB = best;
    }
    pl.n_rowblk = (int)ceil_div(I0, 16 * pl.RB);

    // Column blocks of the output: at most four 16-column blocks per wavefront.
    {
        const int jb_total = (int)ceil_div(R, 16);
        pl.n_jchunk = (int)ceil_div(jb_total, 4);
        pl.JB = (int)ceil_div(jb_total, pl.n_jchunk);
    }

    // Column modes: all but mode 0 and mode k.  Inner = lowest one with at
    // least 8 entries, else the largest; the others are outer modes.
    int cols[MTTKRP_MAX_NDIM];
    int n_cols = 0;
    for (int m = 1; m < ndim; ++m)
        if (m != k)
            cols[n_cols++] = m;
    pl.inner = -1;
    for (int c = 0; c < n_cols; ++c)
        if (dims[cols[c]] >= 8) { pl.inner = cols[c]; break; }
    if (pl.inner < 0)
        for (int c = 0; c < n_cols; ++c)
            if (pl.inner < 0 || dims[cols[c]] > dims[pl.inner])
                pl.inner = cols[c];
    pl.n_out = 0;
    pl.o_total = 1;
    for (int c = 0; c < n_cols; ++c)
        if (cols[c] != pl.inner) {
            pl.out_modes[pl.n_out++] = cols[c];
            pl.o_total *= dims[cols[c]];
        }
    pl.I_in = pl.inner >= 0 ? dims[pl.inner] : 1;
    pl.n_batch = k == 0 ? 1 : (int)dims[k];

    // Split the (outer x inner) column space so that about target_items
    // wavefront items exist, each with enough steps to amortise its epilogue.
    const int64_t steps_in = ceil_div(pl.I_in, 4);
    const int64_t steps_all = pl.o_total * steps_in;
    const int64_t base_items = (int64_t)pl.n_rowblk * pl.n_jchunk * pl.n_batch;
    const int64_t target = tn.target_items > 0 ? tn.target_items : 8192;
    const int64_t min_steps = 16;
    int64_t max_steps = tn.max_steps > 0 ? tn.max_steps
                        : (sbytes == 4 ? 1024 : ((int64_t)1 << 40));   // fp32: short accumulation chains
    int64_t F = ceil_div(target, base_items);
    if (F > steps_all / min_steps)
        F = steps_all / min_steps;
    if (F < 1)
        F = 1;
    if (k == 0) {
        // partial tiles are written once and read once: keep that below ws_percent of X
        const double pct = tn.ws_percent > 0 ? (double)tn.ws_percent : 3.0;
        const double cap = pct * 0.01 * (double)pl.N / (2.0 * (double)I0 * (double)R);
        if ((double)F > cap)
            F = cap < 1.0 ? 1 : (int64_t)cap;
    }
    if (F < ceil_div(steps_all, max_steps))
        F = ceil_div(steps_all, max_steps);
    pl.n_osplit = F < pl.o_total ? F : pl.o_total;
    pl.o_per_item = ceil_div(pl.o_total, pl.n_osplit);
    pl.n_osplit = ceil_div(pl.o_total, pl.o_per_item);
    int64_t F_in = ceil_div(F, pl.n_osplit);
    if (pl.o_per_item > 1)
        F_in = 1;   // inner splitting only once every item is down to one outer iteration
    if (F_in > steps_in)
        F_in = steps_in;
    pl.cols_per_isplit = (int)(4 * ceil_div(steps_in, F_in));
    pl.n_isplit = (int)ceil_div(pl.I_in, pl.cols_per_isplit);
    pl.steps_per_item = pl.o_per_item * (pl.cols_per_isplit / 4);
    if (pl.steps_per_item >= ((int64_t)1 << 30))
        return MTTKRP_ERR_UNSUPPORTED;

    pl.n_items = base_items * pl.n_osplit * pl.n_isplit;
    if (pl.n_items >= ((int64_t)1 << 31) - 64)
        return MTTKRP_ERR_UNSUPPORTED;
    if (k == 0)
        pl.n_slots = pl.n_osplit * pl.n_isplit;
    else
        pl.n_slots = pl.n_osplit * pl.n_isplit * pl.n_rowblk;
    if (pl.n_slots >= ((int64_t)1 << 31))
        return MTTKRP_ERR_UNSUPPORTED;
    pl.ws_bytes = pl.n_slots > 1
        ? (size_t)pl.n_slots * (size_t)dims[k] * (size_t)R * (size_t)sbytes : 0;
    pl.xcd_remap = tn.xcd_remap != 2;
    return MTTKRP_OK;
}

template <typename T, int RB, int JB>
void launch_stream(const StreamArgs<T>& a, dim3 grid, hipStream_t st)
{
    hipLaunchKernelGGL((mttkrp_stream_kernel<T, RB, JB>), grid, dim3(kBlockThreads), 0, st, a);
}

template <typename T, int RB>
void launch_stream_jb(int JB, const StreamArgs<T>& a, dim3 grid, hipStream_t st)
{
    switch (JB) {
    case 1: launch_stream<T, RB, 1>(a, grid, st); break;
    case 2: launch_stream<T, RB, 2>(a, grid, st); break;
    case 3: launch_stream<T, RB, 3>(a, grid, st); break;
    default: launch_stream<T, RB, 4>(a, grid, st); break;
    }
}

template <typename T>
void launch_stream_rb(int RB, int JB, const StreamArgs<T>& a, dim3 grid, hipStream_t st)
{
    switch (RB) {
    case 1: launch_stream_jb<T, 1>(JB, a, grid, st); break;
    case 2: launch_stream_jb<T, 2>(JB, a, grid, st); break;
    case 3: launch_stream_jb<T, 3>(JB, a, grid, st); break;
    default: launch_stream_jb<T, 4>(JB, a, grid, st); break;
    }
}

constexpr int kTimingSlots = 512;   // ring of timed calls kept per device

struct TimedCall {
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};   // stream begin/end, combine begin/end
    bool combine = false;
};

struct DeviceState {
    void* ws = nullptr;
    size_t ws_bytes = 0;
    TimedCall* calls = nullptr;  // kTimingSlots entries once timing has been used
    int64_t n_timed = 0;         // calls recorded since timing was last enabled
};
DeviceState g_dev[kMaxDevices];
bool g_timing = false;

template <typename T>
int run(int ndim, const int64_t* dims, const T* X, const T* const* factors, int R, int k, T* M,
        void* workspace, size_t workspace_bytes, bool own_ws, void* stream)
{
    if (!X || !M || !factors)
        return MTTKRP_ERR_INVALID_ARG;
    Plan pl;
    int rc = make_plan(ndim, dims, R, k, (int)sizeof(T), pl);
    if (rc != MTTKRP_OK)
        return rc;
    for (int m = 0; m < ndim; ++m)
        if (m != k && !factors[m])
            return MTTKRP_ERR_INVALID_ARG;

    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    if (dev < 0 || dev >= kMaxDevices)
        return MTTKRP_ERR_UNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;

    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState& ds = g_dev[dev];
    T* ws = nullptr;
    if (pl.ws_bytes > 0) {
        if (own_ws) {
            if (ds.ws_bytes < pl.ws_bytes) {
                if (ds.ws) {
                    if (hipDeviceSynchronize() != hipSuccess)
                        return MTTKRP_ERR_DEVICE;
                    (void)hipFree(ds.ws);
                    ds.ws = nullptr;
                    ds.ws_bytes = 0;
                }
                size_t want = pl.ws_bytes + (pl.ws_bytes >> 2);
                if (hipMalloc(&ds.ws, want) != hipSuccess) {
                    (void)hipGetLastError();
                    return MTTKRP_ERR_DEVICE;
                }
                ds.ws_bytes = want;
            }
            ws = (T*)ds.ws;
        } else {
            if (!workspace || workspace_bytes < pl.ws_bytes || ((uintptr_t)workspace & 255u))
                return MTTKRP_ERR_WORKSPACE;
            ws = (T*)workspace;
        }
    }
    const bool timing = g_timing;
    TimedCall* tc = nullptr;
    if (timing) {
        if (!ds.calls) {
            TimedCall* calls = new (std::nothrow) TimedCall[kTimingSlots];
            if (!calls)
                return MTTKRP_ERR_DEVICE;
            for (int c = 0; c < kTimingSlots; ++c)
                for (int e = 0; e < 4; ++e)
                    if (hipEventCreate(&calls[c].ev[e]) != hipSuccess) {
                        delete[] calls;   // events created so far are leaked; creation does not fail in practice
                        return MTTKRP_ERR_DEVICE;
                    }
            ds.calls = calls;
        }
        tc = &ds.calls[ds.n_timed % kTimingSlots];
    }

    StreamArgs<T> a;
    memset(&a, 0, sizeof(a));
    a.X = X;
    a.A_row = k == 0 ? nullptr : factors[0];
    a.A_in = pl.inner >= 0 ? factors[pl.inner] : factors[0];   // without column modes k != 0, so factors[0] exists
    a.no_inner = pl.inner >= 0 ? 0 : 1;
    a.sx_in = pl.inner >= 0 ? pl.strides[pl.inner] : 0;
    a.sx_batch = k == 0 ? 0 : pl.strides[k];
    for (int m = 0; m < kMaxOuter; ++m) {
        a.A_out[m] = nullptr;
        a.sx_out[m] = 0;
        a.dim_out[m] = 1;
    }
    for (int m = 0; m < pl.n_out; ++m) {
        a.A_out[m] = factors[pl.out_modes[m]];
        a.sx_out[m] = pl.strides[pl.out_modes[m]];
        a.dim_out[m] = (int32_t)pl.dims[pl.out_modes[m]];
    }
    a.out = pl.n_slots > 1 ? ws : M;
    a.o_total = pl.o_total;
    a.o_per_item = pl.o_per_item;
    a.n_out = pl.n_out;
    a.I0 = (int32_t)pl.dims[0];
    a.I_in = (int32_t)pl.I_in;
    a.R = R;
    a.first_mode = k == 0;
    a.n_rowblk = pl.n_rowblk;
    a.n_jchunk = pl.n_jchunk;
    a.n_batch = pl.n_batch;
    a.n_isplit = pl.n_isplit;
    a.cols_per_isplit = pl.cols_per_isplit;
    a.n_items = (int32_t)pl.n_items;
    a.n_slots = (int32_t)pl.n_slots;
    a.xcd_remap = pl.xcd_remap ? 1 : 0;

    int64_t blocks = ceil_div(pl.n_items, kWaves);
    if (a.xcd_remap)
        blocks = ceil_div(blocks, 8) * 8;
    if (blocks >= ((int64_t)1 << 31))
        return MTTKRP_ERR_UNSUPPORTED;

    (void)hipGetLastError();
    if (timing)
        (void)hipEventRecord(tc->ev[0], st);
    launch_stream_rb<T>(pl.RB, pl.JB, a, dim3((unsigned)blocks), st);
    if (timing) {
        (void)hipEventRecord(tc->ev[1], st);
        tc->combine = false;
    }
    if (hipGetLastError() != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    if (pl.n_slots > 1) {
        const int64_t n_elems = pl.dims[k] * (int64_t)R;
        const int64_t stride_row = k == 0 ? R : pl.n_slots * (int64_t)R;
        const int64_t stride_slot = k == 0 ? pl.dims[0] * (int64_t)R : R;
        if (timing)
            (void)hipEventRecord(tc->ev[2], st);
        hipLaunchKernelGGL((mttkrp_combine_kernel<T>), dim3((unsigned)ceil_div(n_elems, 256)),
                           dim3(256), 0, st, (const T*)ws, M, n_elems, R, (int)pl.n_slots,
                           stride_row, stride_slot);
        if (timing) {
            (void)hipEventRecord(tc->ev[3], st);
            tc->combine = true;
        }
        if (hipGetLastError() != hipSuccess)
            return MTTKRP_ERR_DEVICE;
    }
    if (timing)
        ds.n_timed += 1;
    return MTTKRP_OK;
}

}  // namespace

extern "C" {

int mttkrp_dense_f64(int ndim, const int64_t* dims, const double* X, const double* const* factors,
                     int R, int k, double* M, void* stream)
{
    return run<double>(ndim, dims, X, factors, R, k, M, nullptr, 0, true, stream);
}

int mttkrp_dense_f32(int ndim, const int64_t* dims, const float* X, const float* const* factors,
                     int R, int k, float* M, void* stream)
{
    return run<float>(ndim, dims, X, factors, R, k, M, nullptr, 0, true, stream);
}

size_t mttkrp_dense_workspace_bytes(int ndim, const int64_t* dims, int R, int k, int dtype_bytes)
{
    Plan pl;
    if (make_plan(ndim, dims, R, k, dtype_bytes, pl) != MTTKRP_OK)
        return (size_t)-1;
    return pl.ws_bytes;
}

int mttkrp_dense_f64_ws(int ndim, const int64_t* dims, const double* X,
                        const double* const* factors, int R, int k, double* M, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    return run<double>(ndim, dims, X, factors, R, k, M, workspace, workspace_bytes, false, stream);
}

int mttkrp_dense_f32_ws(int ndim, const int64_t* dims, const float* X, const float* const* factors,
                        int R, int k, float* M, void* workspace, size_t workspace_bytes,
                        void* stream)
{
    return run<float>(ndim, dims, X, factors, R, k, M, workspace, workspace_bytes, false, stream);
}

const char* mttkrp_status_string(int status)
{
    switch (status) {
    case MTTKRP_OK: return "ok";
    case MTTKRP_ERR_INVALID_ARG: return "invalid argument";
    case MTTKRP_ERR_UNSUPPORTED: return "unsupported size or number of modes";
    case MTTKRP_ERR_WORKSPACE: return "workspace too small or misaligned";
    case MTTKRP_ERR_DEVICE: return "HIP runtime call failed";
    default: return "unknown status";
    }
}

int mttkrp_version(void) { return 100; }

void mttkrp_release(void)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    int cur = 0;
    if (hipGetDevice(&cur) != hipSuccess)
        return;
    for (int d = 0; d < kMaxDevices; ++d) {
        DeviceState& ds = g_dev[d];
        if (!ds.ws && !ds.calls)
            continue;
        if (hipSetDevice(d) != hipSuccess)
            continue;
        (void)hipDeviceSynchronize();
        if (ds.ws)
            (void)hipFree(ds.ws);
        ds.ws = nullptr;
        ds.ws_bytes = 0;
        if (ds.calls) {
            for (int c = 0; c < kTimingSlots; ++c)
                for (int e = 0; e < 4; ++e)
                    (void)hipEventDestroy(ds.calls[c].ev[e]);
            delete[] ds.calls;
        }
        ds.calls = nullptr;
        ds.n_timed = 0;
    }
    (void)hipSetDevice(cur);
}

int mttkrp_timing_enable(int enable)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_timing = enable != 0;
    if (g_timing)
        for (int d = 0; d < kMaxDevices; ++d)
            g_dev[d].n_timed = 0;
    return MTTKRP_OK;
}

int64_t mttkrp_timing_count(void)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return 0;
    std::lock_guard<std::mutex> lock(g_mutex);
    return g_dev[dev].n_timed;
}

int mttkrp_timing_get(int64_t index, float* stream_ms, float* combine_ms)
{
    if (!stream_ms || !combine_ms)
        return MTTKRP_ERR_INVALID_ARG;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    if (dev < 0 || dev >= kMaxDevices)
        return MTTKRP_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_mutex);
    DeviceState& ds = g_dev[dev];
    if (!ds.calls || index < 0 || index >= ds.n_timed || index < ds.n_timed - kTimingSlots)
        return MTTKRP_ERR_INVALID_ARG;
    TimedCall& tc = ds.calls[index % kTimingSlots];
    *combine_ms = 0.0f;
    if (hipEventSynchronize(tc.combine ? tc.ev[3] : tc.ev[1]) != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    if (hipEventElapsedTime(stream_ms, tc.ev[0], tc.ev[1]) != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    if (tc.combine && hipEventElapsedTime(combine_ms, tc.ev[2], tc.ev[3]) != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    return MTTKRP_OK;
}

int mttkrp_timing_last(float* stream_ms, float* combine_ms)
{
    return mttkrp_timing_get(mttkrp_timing_count() - 1, stream_ms, combine_ms);
}

int mttkrp_tune_set(const char* key, int64_t value)
{
    if (!key || value < 0)
        return MTTKRP_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!strcmp(key, "row_blocks")) {
        if (value > 4) return MTTKRP_ERR_INVALID_ARG;
        g_tune.row_blocks = value;
    } else if (!strcmp(key, "target_items")) {
        g_tune.target_items = value;
    } else if (!strcmp(key, "max_steps")) {
        g_tune.max_steps = value;
    } else if (!strcmp(key, "xcd_remap")) {
        if (value > 2) return MTTKRP_ERR_INVALID_ARG;
        g_tune.xcd_remap = value;
    } else if (!strcmp(key, "ws_percent")) {
        if (value > 100) return MTTKRP_ERR_INVALID_ARG;
        g_tune.ws_percent = value;
    } else {
        return MTTKRP_ERR_INVALID_ARG;
    }
    return MTTKRP_OK;
}

int mttkrp_plan_describe(int ndim, const int64_t* dims, int R, int k, int dtype_bytes, char* buf,
                         size_t buflen)
{
    if (!buf || buflen == 0)
        return MTTKRP_ERR_INVALID_ARG;
    buf[0] = 0;
    Plan pl;
    int rc = make_plan(ndim, dims, R, k, dtype_bytes, pl);
    if (rc != MTTKRP_OK)
        return rc;
    snprintf(buf, buflen,
             "shape=%s rows_per_wave=%d row_blocks=%d col_blocks=%d j_chunks=%d inner_mode=%d "
             "outer_modes=%d batch=%d o_per_item=%lld outer_splits=%lld inner_splits=%d "
             "items=%lld steps_per_item=%lld slots=%lld ws_bytes=%zu",
             k == 0 ? "first" : (k == ndim - 1 ? "last" : "middle"), 16 * pl.RB, pl.n_rowblk,
             pl.JB, pl.n_jchunk, pl.inner, pl.n_out, pl.n_batch, (long long)pl.o_per_item,
             (long long)pl.n_osplit, pl.n_isplit, (long long)pl.n_items,
             (long long)pl.steps_per_item, (long long)pl.n_slots, pl.ws_bytes);
    return MTTKRP_OK;
}

}  // extern "C"
