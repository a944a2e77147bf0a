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
#ifndef MTTKRP_ASM_PIPE
#define MTTKRP_ASM_PIPE 1
#endif
#ifndef MTTKRP_DEPTH
#define MTTKRP_DEPTH 4
#endif

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


// ---------------------------------------------------------------------------
// Software-pipelined run for fp64 with 4 row blocks x 2 column blocks (R in
// 17..32, the memory-bound flagship case).  The compiler places its waits for
// outstanding loads conservatively around control flow, which keeps a wavefront
// from overlapping its own loads with its own MFMAs; this hand-scheduled loop
// keeps several steps of loads in flight while the MFMAs of an earlier one run.  It
// covers any run of at least that many consecutive unmasked steps of one sweep: X pointer
// and factor offsets advance by constant strides, one weight Q per column block.
// Temporaries live in fixed registers (declared as clobbers); the loads of step
// t go to operand set t modulo the ring size; every wait names how many later
// loads may still be outstanding (memory operations return in issue order).
#include "mttkrp_pipe.inc"

template <bool NT>
__device__ __forceinline__ void pipelined_run_d42(double4_t (&acc)[4][2], const double*& xq,
                                                  int64_t x_step_bytes, const double* bbase,
                                                  uint32_t bo, uint32_t b_step_bytes,
                                                  double q0, double q1, int n_more)
{
#define MTTKRP_PIPE_D42_OPERANDS                                                                   \
    [xq] "+v"(xq), [bo] "+v"(bo), [n] "+s"(n_more), [a00] "+v"(acc[0][0]),      \
        [a01] "+v"(acc[0][1]), [a10] "+v"(acc[1][0]), [a11] "+v"(acc[1][1]), [a20] "+v"(acc[2][0]), \
        [a21] "+v"(acc[2][1]), [a30] "+v"(acc[3][0]), [a31] "+v"(acc[3][1])                         \
        : [xs] "s"(x_step_bytes), [bb] "s"(bbase), [bs] "s"(b_step_bytes), [q0] "v"(q0), [q1] "v"(q1) \
        : MTTKRP_PIPE_D42_CLOBBERS
    if (NT)
        asm volatile(MTTKRP_PIPE_D42_ASM_NT : MTTKRP_PIPE_D42_OPERANDS);
    else
        asm volatile(MTTKRP_PIPE_D42_ASM : MTTKRP_PIPE_D42_OPERANDS);
#undef MTTKRP_PIPE_D42_OPERANDS
}

template <typename T, int RB, int JB> struct HasPipe { static constexpr bool value = false; };
#if MTTKRP_ASM_PIPE
template <> struct HasPipe<double, 4, 2> { static constexpr bool value = true; };
#endif

// Generic stand-in so that the call below compiles for every instantiation.
template <bool NT, typename T, int RB, int JB>
__device__ __forceinline__ void pipelined_run(typename Mfma<T>::acc_t (&acc)[RB][JB], const T*& xq,
                                              int64_t x_step_bytes, const T* bbase, uint32_t bo,
                                              uint32_t b_step_bytes, T q0, T q1, int n_more)
{
    if constexpr (HasPipe<T, RB, JB>::value)
        pipelined_run_d42<NT>(acc, xq, x_step_bytes, bbase, bo, b_step_bytes, q0, q1, n_more);
}

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
    int32_t n_splits;            // column-space splits (outer splits x inner splits)
    int32_t xcd_remap;
    int32_t group4;              // first mode: 1 = four wavefronts per partial tile (LDS sum)
    int32_t no_inner;            // 1: no column mode at all; A_in is only a readable dummy
#ifdef MTTKRP_TRACE
    long long* trace;            // debug builds: four clock readings per work item, or null
#endif
};


// How the N 16-wide MFMA blocks of a wavefront tile map to rows (or output
// columns).  A lane feeds MFMA index m of every block, so giving it N consecutive
// rows lets one wide load instruction fetch its entries for all N blocks: block b
// holds rows N*m + b.  A load instruction carries at most 16 bytes per lane, so
// more than 16 bytes are split into two chunks of n0 and n1 blocks; chunk 0 covers
// the first 16*n0 rows, chunk 1 the next 16*n1, and within each chunk every
// 16-lane group still reads one contiguous piece of memory.
template <typename T, int N> struct Lay {
    static constexpr int G = 16 / (int)sizeof(T);
    static constexpr int n0 = N < G ? N : G;
    static constexpr int n1 = N - n0;
    static_assert(n1 <= G, "at most two chunks");
    // offset of block b's entry for MFMA index m from the tile's first row (column)
    static __device__ __forceinline__ int off(int b, int m)
    {
        return b < n0 ? n0 * m + b : 16 * n0 + n1 * m + (b - n0);
    }
};

// Load of a tensor entry.  When every 16-row segment a load instruction reads is
// a whole, aligned 128-byte line (fp64, I_0 a multiple of 16, aligned X), the line
// is never needed again and a non-temporal load keeps it from displacing the
// factor rows in L2.  Otherwise neighbouring load instructions share lines
// (fp32 segments are half lines, unaligned segments straddle two), and the
// line has to stay cacheable until its other half has been read.
template <bool NT, typename T> __device__ __forceinline__ T stream_load(const T* p)
{
    if (NT)
        return __builtin_nontemporal_load(p);
    return *p;
}

// n consecutive values; the compiler merges them into one wide load instruction
template <bool NT, int N, typename T> __device__ __forceinline__ void load_vec(const T* p, T* out)
{
#pragma unroll
    for (int i = 0; i < N; ++i)
        out[i] = stream_load<NT>(p + i);
}
// Rows use the same scheme in fp32 and for three fp64 row blocks.  With two or
// four fp64 row blocks every row block keeps a load instruction of its own (block
// b holds rows 16*b + m, 8 bytes per lane): measured on 1024- and 16384-row
// tensors, 16-byte non-temporal tensor loads cost 3 to 15 % of the bandwidth there.
template <typename T, int N> struct LayRows : Lay<T, N> {};
#ifndef MTTKRP_F64_WIDE_ROWS
#define MTTKRP_F64_WIDE_ROWS 0      // 1: 16-byte tensor loads for every fp64 tile (experiments)
#endif
#if !MTTKRP_F64_WIDE_ROWS
template <> struct LayRows<double, 2> {
    static constexpr int n0 = 1;
    static constexpr int n1 = 0;
    static __device__ __forceinline__ int off(int b, int m) { return 16 * b + m; }
};
template <> struct LayRows<double, 4> : LayRows<double, 2> {};
#endif

// the entries of one lane for all N row blocks; d1 = lane offset of chunk 1
template <bool NT, int N, typename T>
__device__ __forceinline__ void load_blocks(const T* p, int d1, T* out)
{
    typedef LayRows<T, N> L;
    if constexpr (L::n0 == 1 && L::n1 == 0 && N > 1) {
#pragma unroll
        for (int b = 0; b < N; ++b)
            out[b] = stream_load<NT>(p + 16 * b);
    } else {
        load_vec<NT, L::n0>(p, out);
        if constexpr (L::n1 > 0)
            load_vec<NT, L::n1>(p + d1, out + L::n0);
    }
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int64_t uni64(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Register budget of one instantiation (fitted to what the compiler allocates):
// accumulators take RB*JB*4 values, every step of a batch RB + 2*JB values (X,
// factor entries, weights), and the rest is about 22 + 20*JB registers in fp64,
// 26 + 11*JB in fp32.  Aim for four wavefronts per SIMD (128 registers) when four
// steps per batch still fit, else three (168 registers) with at least two
// steps, else two (256 registers).
template <typename T, int RB, int JB> struct Budget {
    static constexpr int w = (int)sizeof(T) / 4;                 // registers per value
    static constexpr int acc = RB * JB * 4 * w;
    static constexpr int fixed = w == 2 ? 22 + 20 * JB : 26 + 11 * JB;
    static constexpr int per_step = (RB + 2 * JB) * w;
    static constexpr int fit(int regs) { return (regs - fixed - acc) / per_step; }
    static constexpr int waves = fit(128 + 8) >= 4 ? 4 : (fit(168 + 8) >= 2 ? 3 : 2);
    static constexpr int raw = waves == 4 ? fit(128 + 8) : (waves == 3 ? fit(168 + 8) : fit(256));
    static constexpr int steps = raw > MTTKRP_DEPTH ? MTTKRP_DEPTH : (raw < 2 ? 2 : raw);
};

// One wavefront = one work item = (row block, column-block chunk, batch value,
// inner split, outer split).  No LDS, no barriers.
//
// Outer column modes: the first one ("mid") is walked by a plain counter; the
// others ("far") only change when mid wraps, and are then re-derived from the
// linear outer index by division (rare).
template <typename T, int RB, int JB, bool NT>
__global__ void __launch_bounds__(kBlockThreads, (HasPipe<T, RB, JB>::value ? MTTKRP_PIPE_D42_WAVES : Budget<T, RB, JB>::waves))
mttkrp_stream_kernel(const StreamArgs<T> p)
{
    // steps per batch = steps of loads in flight; where the hand-scheduled run takes the bulk
    // of the steps, short batches leave the registers to it
    constexpr int U = HasPipe<T, RB, JB>::value ? 2 : Budget<T, RB, JB>::steps;
    typedef Mfma<T> MF;
    typedef typename MF::acc_t acc_t;

    const int lane = threadIdx.x & 63;
    const int wave = uni((int)(threadIdx.x >> 6));
    uint32_t blk = blockIdx.x;
    if (p.xcd_remap)   // workgroups go round-robin over the 8 XCDs: give each XCD a contiguous range
        blk = (blk & 7u) * (gridDim.x >> 3) + (blk >> 3);
    // Item decode.  First mode: the four wavefronts of a workgroup share (row
    // block, column chunk) and take four consecutive column-space splits, so that
    // their tiles can be summed in LDS; a whole workgroup is in range or not.
    // Other modes: one independent item per wavefront.
    const bool grouped = p.first_mode && p.group4;   // four wavefronts sum their tiles in LDS
    uint32_t it = grouped ? blk : blk * kWaves + wave;
#ifdef MTTKRP_TRACE
    const uint32_t trace_item = blk * kWaves + wave;
    long long trace_t[4];
    trace_t[0] = (long long)__builtin_readcyclecounter();
#endif
    if (it >= (uint32_t)(grouped ? p.n_items / kWaves : p.n_items))
        return;
    const int rowblk = uni((int)(it % (uint32_t)p.n_rowblk));  it /= (uint32_t)p.n_rowblk;
    const int jchunk = uni((int)(it % (uint32_t)p.n_jchunk));  it /= (uint32_t)p.n_jchunk;
    const int batch = uni((int)(it % (uint32_t)p.n_batch));    it /= (uint32_t)p.n_batch;
    const int group = uni((int)it);                             // first mode: split group (or split)
    const uint32_t sp = grouped ? it * kWaves + wave : it;        // column-space split
    const bool empty = sp >= (uint32_t)p.n_splits;              // padding of the last split group
    const int osp = empty ? 0 : uni((int)(sp / (uint32_t)p.n_isplit));
    const int isp = empty ? 0 : uni((int)(sp - (uint32_t)osp * (uint32_t)p.n_isplit));

    typedef LayRows<T, RB> LR;  // rows of the RB row blocks
    typedef Lay<T, JB> LC;      // output columns of the JB column blocks
    const int il = lane & 15;   // MFMA index of this lane: row index for operand A, column index for B and D
    const int kk = lane >> 4;   // which of the step's four columns this lane feeds
    const int R = p.R;

    // Rows: the last row block is shifted down to end at I0 so that every load
    // stays inside the tensor; rows it shares with the previous block are
    // dropped in the epilogue.  With fewer than 16 rows lanes clamp instead.
    const int first_row = rowblk * (16 * RB);
    int row_base = first_row;
    if (row_base + 16 * RB > p.I0)
        row_base = p.I0 > 16 * RB ? p.I0 - 16 * RB : 0;
    const int lrow = min(LR::n0 * il, p.I0 - LR::n0 - row_base);        // this lane's first row in the tile (chunk 0)
    const int xd1 = 16 * LR::n0 + (LR::n1 - LR::n0) * il;              // from there to its first row of chunk 1

    // Columns of the output (j).  A lane holds LC::n0 consecutive columns (and LC::n1 more of
    // chunk 1).  Where such a group would cross R it is moved back to end at R, so that every
    // load stays inside the factor rows; the columns it then shares with a lower lane are
    // computed twice and stored by their owner only.
    const int j_first = jchunk * (16 * JB);
    const int jt0 = j_first + LC::n0 * il;
    const int jt1 = j_first + 16 * LC::n0 + LC::n1 * il;
    const int js0 = min(jt0, R - LC::n0);
    const int js1 = LC::n1 > 0 ? min(jt1, R - LC::n1) : 0;
    int jc[JB];          // column of block jb in this lane
    bool jown[JB];       // and whether this lane stores it
#pragma unroll
    for (int jb = 0; jb < JB; ++jb) {
        jc[jb] = jb < LC::n0 ? js0 + jb : js1 + (jb - LC::n0);
        jown[jb] = jb < LC::n0 ? jc[jb] >= jt0 : jc[jb] >= jt1;
    }
    auto load_cols = [&](const T* row, T (&out)[JB]) {     // entries of a factor row at this lane's columns
        load_vec<false, LC::n0>(row + js0, out);
        if constexpr (LC::n1 > 0)
            load_vec<false, LC::n1>(row + js1, out + LC::n0);
    };

    // Range of this item in the (outer iteration, inner column) space.
    const int ia_begin = isp * p.cols_per_isplit;
    const int ia_end = min(p.I_in, ia_begin + p.cols_per_isplit);
    const int steps_in = (ia_end - ia_begin + 3) >> 2;
    const int64_t o_begin = (int64_t)osp * p.o_per_item;
    const int o_count = empty ? 0 : uni((int)min(p.o_per_item, p.o_total - o_begin));

    const T* const xlane = p.X + (int64_t)batch * p.sx_batch + (row_base + lrow);
    const int64_t x_step = 4 * p.sx_in;
    const bool no_inner = p.no_inner != 0;   // then A_in is a readable dummy and b = 1
    const int dim_mid = p.dim_out[0];        // 1 when there is no outer mode
    const int64_t sx_mid = p.sx_out[0];
    const bool has_mid = p.n_out > 0;
    const T* const A_mid = has_mid ? p.A_out[0] : p.A_in;   // dummy when unused

    // Last step of a sweep: lanes whose column lies beyond the inner range read
    // the sweep's last column instead and get weight 0.  How many lanes that is
    // depends only on the item, not on the step.
    const int over = max(kk - ((ia_end - ia_begin - 1) & 3), 0);
    const bool lane_ok = over == 0;
    const int64_t x_back = (int64_t)over * p.sx_in;
    const int64_t b_back = (int64_t)over * R;   // bbase is per-lane in the last step only

    // State of the outer walk (all wave-uniform except the factor values).
    int i_mid = 0;
    int i_far[kMaxOuter];         // i_far[m] for outer modes m >= 1
    int64_t xoff_far = 0;         // X offset of the far modes
    T Qfar[JB];                   // product of the far modes' factor entries
    T Q[JB];                      // ... times the mid mode's entry: weight of the sweep being issued
    auto load_far = [&]() {       // Qfar from the current far indices (rare)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            Qfar[jb] = (T)1;
#pragma unroll
        for (int m = 1; m < kMaxOuter; ++m) {
            if (m < p.n_out) {
                T a[JB];
                load_cols(p.A_out[m] + (int64_t)i_far[m] * R, a);
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
                    Qfar[jb] *= a[jb];
            }
        }
    };
    auto load_Q = [&]() {         // Q of the sweep the cursor enters
        T a[JB];
        load_cols(A_mid + (int64_t)(has_mid ? i_mid : 0) * R, a);
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            Q[jb] = has_mid ? Qfar[jb] * a[jb] : Qfar[jb];
    };
#pragma unroll
    for (int m = 0; m < kMaxOuter; ++m)
        i_far[m] = 0;
    if (o_begin > 0) {   // decode the first outer index of this item (the only divisions of the walk)
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
    load_Q();

    // Cursor of the issue side: it points at the next step to issue.
    int s_in = 0;                       // step inside the current sweep
    const T* xp = xlane + xoff_far + (int64_t)i_mid * sx_mid + (int64_t)(ia_begin + kk) * p.sx_in;
    const T* bbase = p.A_in + (int64_t)ia_begin * R;            // wave-uniform: factor row of the step's first column
    // per-lane byte offsets of (column kk, first output column of chunk 0 / chunk 1)
    const uint32_t boff0 = ((uint32_t)kk * (uint32_t)R + (uint32_t)js0) * (uint32_t)sizeof(T);
    const uint32_t boff1 = ((uint32_t)kk * (uint32_t)R + (uint32_t)js1) * (uint32_t)sizeof(T);
    auto load_b = [&](const char* row, T (&out)[JB]) {      // factor entries of one step
        load_vec<false, LC::n0>((const T*)(row + boff0), out);
        if constexpr (LC::n1 > 0)
            load_vec<false, LC::n1>((const T*)(row + boff1), out + LC::n0);
    };
    const int n_steps = o_count * steps_in;   // < 2^30, checked on the host
    int remaining = n_steps;        // steps not yet issued, the cursor's included
    bool parked = false;                // all steps issued: the cursor stays on the last one, weight 0
    // Steps that need no lane masking: all of a sweep when its length is a multiple of four
    // columns, else all but the last.
    const int steps_plain = ((ia_end - ia_begin) & 3) == 0 ? steps_in : steps_in - 1;

    auto next_sweep = [&]() {           // wave-uniform, once per inner sweep
        s_in = 0;
        bbase = p.A_in + (int64_t)ia_begin * R;
        i_mid += 1;
        if (i_mid >= dim_mid) {         // mid wraps: carry into the far modes
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
        }
        load_Q();
        xp = xlane + xoff_far + (int64_t)i_mid * sx_mid + (int64_t)(ia_begin + kk) * p.sx_in;
    };
    // Generic single step: issue the loads of the cursor's step into one operand set ...
    auto issue = [&](T (&xn)[RB], T (&bn)[JB], T (&qn)[JB]) {
        const bool last = s_in == steps_in - 1;           // wave-uniform
        const T* xe = last ? xp - x_back : xp;
        const char* be = (const char*)(last ? bbase - b_back : bbase);
        load_blocks<NT, RB>(xe, xd1, xn);
        load_b(be, bn);
        if (no_inner) {
#pragma unroll
            for (int jb = 0; jb < JB; ++jb)
                bn[jb] = (T)1;
        }
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            qn[jb] = (parked || (last && !lane_ok)) ? (T)0 : Q[jb];
    };
    // ... and move the cursor one step on.
    auto advance = [&]() {
        remaining -= 1;
        if (remaining <= 0) {
            parked = true;
            return;
        }
        s_in += 1;
        if (s_in < steps_in) {
            xp += x_step;
            bbase += 4 * (int64_t)R;
        } else {
            next_sweep();
        }
    };

    acc_t acc[RB][JB];
#pragma unroll
    for (int r = 0; r < RB; ++r)
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            acc[r][jb] = (acc_t)(0);

    // Steps are taken in batches of U: first all loads of the batch are issued
    // (U steps of X and factor rows in flight per wavefront), then the MFMAs of
    // the U steps run in issue order, each waiting only for its own operands.
    // Other wavefronts of the SIMD fill the gaps between batches.
    //   plain batch:   U unmasked steps of one sweep: one weight Q, constant strides
    //   generic batch: any steps (sweep boundaries, masked last step, parked padding)
#ifdef MTTKRP_TRACE
    trace_t[1] = (long long)__builtin_readcyclecounter();
#endif
    // the pipelined run addresses the inner factor with 32-bit offsets
    const bool pipe_ok = HasPipe<T, RB, JB>::value && (int64_t)p.I_in * R * (int64_t)sizeof(T) < ((int64_t)1 << 31);
    int done = 0;
    while (done < n_steps) {
        if (HasPipe<T, RB, JB>::value) {
            const int avail = parked || !pipe_ok ? 0 : min(remaining, steps_plain - s_in);
            if (avail >= MTTKRP_PIPE_D42_DEPTH) {
                const int n_run = avail;
                pipelined_run<NT, T, RB, JB>(acc, xp, x_step * (int64_t)sizeof(T), bbase, boff0,
                                             4u * (uint32_t)R * (uint32_t)sizeof(T),
                                             Q[0], Q[JB > 1 ? 1 : 0], avail - MTTKRP_PIPE_D42_DEPTH);
                bbase += (int64_t)n_run * 4 * R;
                s_in += n_run;
                remaining -= n_run;
                done += n_run;
                if (remaining <= 0) {   // park on the run's last step
                    parked = true;
                    s_in -= 1;
                    xp -= x_step;
                    bbase -= 4 * (int64_t)R;
                } else if (s_in >= steps_in) {
                    next_sweep();
                }
                continue;
            }
        }
        T xs[U][RB], bs[U][JB], qs[U][JB];
        done += U;
        if (!parked && remaining >= U && s_in + U <= steps_plain) {
            const T* xu = xp;
            const char* bu = (const char*)bbase;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                load_blocks<NT, RB>(xu, xd1, xs[u]);
                load_b(bu, bs[u]);
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
                    qs[u][jb] = Q[jb];
                xu += x_step;
                bu += 4 * (int64_t)R * (int64_t)sizeof(T);
            }
            remaining -= U;
            if (remaining <= 0) {       // park on the batch's last step
                parked = true;
                s_in += U - 1;
                xp += (U - 1) * x_step;
                bbase += (U - 1) * 4 * (int64_t)R;
            } else {
                s_in += U;
                xp += U * x_step;
                bbase += U * 4 * (int64_t)R;
                if (s_in >= steps_in)
                    next_sweep();
            }
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                issue(xs[u], bs[u], qs[u]);
                advance();
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            T bc[JB];
#pragma unroll
            for (int jb = 0; jb < JB; ++jb)
                bc[jb] = bs[u][jb] * qs[u][jb];
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
                    acc[r][jb] = MF::run(xs[u][r], bc[jb], acc[r][jb]);
        }
    }

#ifdef MTTKRP_TRACE
    trace_t[2] = (long long)__builtin_readcyclecounter();
#endif
    // Epilogue.
    if (p.first_mode && !grouped) {
        T* o = p.out + (int64_t)group * ((int64_t)p.I0 * R);
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int row = row_base + LR::off(r, MF::row(lane, q));
                    if (row >= first_row && row < p.I0 && jown[jb])
                        o[(int64_t)row * R + jc[jb]] = acc[r][jb][q];
                }
    } else if (p.first_mode) {
        // Sum the four wavefronts' tiles in LDS in a fixed order, (w0 + w2) + (w1 + w3);
        // all hold the same (row, column) entries in the same registers.
        extern __shared__ unsigned char lds_raw[];
        T* lds = reinterpret_cast<T*>(lds_raw);
        constexpr int kTile = RB * JB * 4 * 64;          // values per wavefront tile
        if (wave >= 2) {
            T* dst = lds + (wave - 2) * kTile + lane;
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        dst[((r * JB + jb) * 4 + q) * 64] = acc[r][jb][q];
        }
        __syncthreads();
        if (wave < 2) {
            const T* src = lds + wave * kTile + lane;
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        acc[r][jb][q] += src[((r * JB + jb) * 4 + q) * 64];
        }
        __syncthreads();
        if (wave == 1) {
            T* dst = lds + lane;
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        dst[((r * JB + jb) * 4 + q) * 64] = acc[r][jb][q];
        }
        __syncthreads();
        if (wave == 0) {
            const T* src = lds + lane;
            T* o = p.out + (int64_t)group * ((int64_t)p.I0 * R);
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int jb = 0; jb < JB; ++jb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const T v = acc[r][jb][q] + src[((r * JB + jb) * 4 + q) * 64];
                        const int row = row_base + LR::off(r, MF::row(lane, q));
                        if (row >= first_row && row < p.I0 && jown[jb])
                            o[(int64_t)row * R + jc[jb]] = v;
                    }
        }
    } else {
        const int64_t slot = ((int64_t)osp * p.n_isplit + isp) * p.n_rowblk + rowblk;
        T* o = p.out + ((int64_t)batch * p.n_slots + slot) * R;
        // Weighted sum over the tile's rows: M(i_k, j) += sum_r A_0(r, j) T(r, j).  The weights
        // of a group of row blocks are all loaded before any is used (one round trip to L2 per
        // group); rows this item does not own (overlap of the shifted last block) get weight 0.
        constexpr int RG = 64 / (4 * JB * (int)(sizeof(T) / 4)) < 1 ? 1 : 64 / (4 * JB * (int)(sizeof(T) / 4));
        double v[JB];
#pragma unroll
        for (int jb = 0; jb < JB; ++jb)
            v[jb] = 0.0;
#pragma unroll
        for (int r0 = 0; r0 < RB; r0 += RG) {
            T w[RG][4][JB];
#pragma unroll
            for (int rr = 0; rr < RG; ++rr)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (r0 + rr < RB) {
                        const int row = row_base + LR::off(r0 + rr, MF::row(lane, q));
                        load_cols(p.A_row + (int64_t)min(row, p.I0 - 1) * R, w[rr][q]);
                    }
#pragma unroll
            for (int rr = 0; rr < RG; ++rr)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int jb = 0; jb < JB; ++jb)
                        if (r0 + rr < RB)
                            asm volatile("" : "+v"(w[rr][q][jb]));   // keeps the loads unconditional and ahead of the sums
#pragma unroll
            for (int rr = 0; rr < RG; ++rr)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (r0 + rr < RB) {
                        const int row = row_base + LR::off(r0 + rr, MF::row(lane, q));
                        const bool ok = row >= first_row && row < p.I0;
#pragma unroll
                        for (int jb = 0; jb < JB; ++jb) {
                            const double t = (double)acc[r0 + rr][jb][q] * (double)w[rr][q][jb];
                            v[jb] += ok ? t : 0.0;
                        }
                    }
        }
#pragma unroll
        for (int jb = 0; jb < JB; ++jb) {
            double t = v[jb];
            t += __shfl_xor(t, 16);
            t += __shfl_xor(t, 32);
            if (kk == 0 && jown[jb])
                o[jc[jb]] = (T)t;
        }
    }
#ifdef MTTKRP_TRACE
    trace_t[3] = (long long)__builtin_readcyclecounter();
    if (p.trace && lane == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            p.trace[(int64_t)trace_item * 4 + i] = trace_t[i];
    }
#endif
}

// M(n, j) = sum of the partial sums of all slots, in fp64 and in a fixed order:
// 16 threads share one output entry, thread q adds slots q, q+16, ... in
// increasing order, then the 16 subtotals are added in order of q.  A block
// covers 16 consecutive entries, so each slot is read in contiguous pieces.
template <typename T>
__global__ void __launch_bounds__(256)
mttkrp_combine_kernel(const T* __restrict__ ws, T* __restrict__ M, int64_t n_elems, int R,
                      int n_slots, int64_t stride_row, int64_t stride_slot,
                      const T* __restrict__ lambda, double beta)
{
    __shared__ double part[16][17];
    const int el = threadIdx.x & 15;
    const int sl = threadIdx.x >> 4;
    const int64_t e = (int64_t)blockIdx.x * 16 + el;
    double s = 0.0;
    if (e < n_elems) {
        const int64_t n = e / R;
        const int j = (int)(e - n * R);
        const T* src = ws + n * stride_row + j;
        int t = sl;
        for (; t + 48 < n_slots; t += 64) {
            const double v0 = (double)src[(int64_t)t * stride_slot];
            const double v1 = (double)src[(int64_t)(t + 16) * stride_slot];
            const double v2 = (double)src[(int64_t)(t + 32) * stride_slot];
            const double v3 = (double)src[(int64_t)(t + 48) * stride_slot];
            s += v0;
            s += v1;
            s += v2;
            s += v3;
        }
        for (; t < n_slots; t += 16)
            s += (double)src[(int64_t)t * stride_slot];
    }
    part[sl][el] = s;
    __syncthreads();
    if (sl == 0 && e < n_elems) {
        double v = 0.0;
#pragma unroll
        for (int q = 0; q < 16; ++q)
            v += part[q][el];
        if (lambda)                      // Eq. (krp): ... diag(lambda)
            v *= (double)lambda[e % R];
        if (beta != 0.0)                 // M is read only when it is accumulated into
            v += beta * (double)M[e];
        M[e] = (T)v;
    }
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
    int64_t max_col_blocks = 0;
    int64_t first_group = 0;
    int64_t waves_per_simd = 0;
    int64_t nt_loads = 0;
#ifdef MTTKRP_TRACE
    int64_t trace_ptr = 0;      // debug builds: device buffer of 4 * n_items int64 clock readings
#endif
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
    int64_t n_splits = 1;      // column-space splits
    int64_t steps_per_item = 0;
    size_t ws_bytes = 0;
    bool xcd_remap = true;
    int group = 4;             // first mode: wavefronts per partial tile
    int wave_cap = 0;          // > 0: resident wavefronts per SIMD are capped (by reserving LDS)
    bool nt_off = false;       // never use non-temporal tensor loads
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
        // fp64 accumulators of more than 12 MFMA tiles do not fit the register file next to the operands
        const int jb_all = (int)ceil_div(ceil_div(R, 16), ceil_div(ceil_div(R, 16), 4));
        const int rb_cap = sbytes == 8 && jb_all == 4 ? 3 : 4;
        const int rb_max = I0 >= 16 ? (int)(I0 / 16 < rb_cap ? I0 / 16 : rb_cap) : 1;
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
        const int cb_max = tn.max_col_blocks >= 1 && tn.max_col_blocks <= 4 ? (int)tn.max_col_blocks : 4;
        pl.n_jchunk = (int)ceil_div(jb_total, cb_max);
        pl.JB = (int)ceil_div(jb_total, pl.n_jchunk);
    }

    // Column modes: all but mode 0 and mode k.  Inner = lowest one with at
    // least 32 entries (eight steps per sweep), else the largest; the others are outer modes.
    int cols[MTTKRP_MAX_NDIM];
    int n_cols = 0;
    for (int m = 1; m < ndim; ++m)
        if (m != k)
            cols[n_cols++] = m;
    pl.inner = -1;
    for (int c = 0; c < n_cols; ++c)
        if (dims[cols[c]] >= 32) { pl.inner = cols[c]; break; }
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
    const int64_t target = tn.target_items > 0 ? tn.target_items : 12288;   // four per resident wavefront slot at three per SIMD
    const int64_t min_steps = 16;
    int64_t max_steps = tn.max_steps > 0 ? tn.max_steps
                        : (sbytes == 4 ? 1024 : ((int64_t)1 << 40));   // fp32: short accumulation chains
    int64_t F = ceil_div(target, base_items);
    if (F > steps_all / min_steps)
        F = steps_all / min_steps;
    if (F < 1)
        F = 1;
    if (k == 0) {
        // One partial tile per workgroup (four splits) is written once and read once: keep
        // that traffic below ws_percent of the bytes of X, or 32 MiB if that is more.
        const double pct = tn.ws_percent > 0 ? (double)tn.ws_percent : 2.0;
        double budget = pct * 0.01 * (double)pl.N * sbytes;
        if (budget < 32.0 * 1048576.0)
            budget = 32.0 * 1048576.0;
        // The hand-scheduled fp64 instantiation gains more from fewer, longer items than from
        // the shared partial tile; every other one is faster with the LDS sum.
        const bool long_items = MTTKRP_ASM_PIPE && sbytes == 8 && pl.RB == 4 && pl.JB == 2;
        pl.group = tn.first_group == 1 ? 1 : tn.first_group == 4 ? kWaves : (long_items ? 1 : kWaves);
        const double cap = pl.group * budget / (2.0 * (double)I0 * (double)R * sbytes);
        if ((double)F > cap)
            F = cap < 1.0 ? 1 : (int64_t)cap;
    }
    if (F < ceil_div(steps_all, max_steps))
        F = ceil_div(steps_all, max_steps);
    if (F < ceil_div(pl.o_total, (int64_t)1 << 29))
        F = ceil_div(pl.o_total, (int64_t)1 << 29);
    // F = outer splits x inner splits.  Among up to eight inner splits (each at least eight
    // steps long) take the pair whose largest item is closest to the average item.
    {
        double best_eff = -1.0;
        for (int64_t ni = 1; ni <= 8; ++ni) {
            if (ni > 1 && steps_in / ni < 8)
                break;
            int64_t no = F / ni;
            if (no < 1)
                no = 1;
            if (no > pl.o_total)
                no = pl.o_total;
            if (ni * pl.o_total < F && ni < 8 && steps_in / (ni + 1) >= 8)
                continue;     // even every sweep on its own is too few: split the inner mode further
            const int64_t opi = ceil_div(pl.o_total, no);
            no = ceil_div(pl.o_total, opi);
            const int64_t in_steps = ceil_div(steps_in, ni);
            const int64_t n_in = ceil_div(pl.I_in, 4 * in_steps);
            const double avg = (double)steps_all / (double)(no * n_in);
            double eff = avg / (double)(opi * in_steps);
            const double ratio = (double)(no * n_in) / (double)F;    // stay near the wanted count
            if (ratio < 0.75)
                eff *= ratio / 0.75;
            if (eff > best_eff + 1e-9) {
                best_eff = eff;
                pl.n_osplit = no;
                pl.o_per_item = opi;
                pl.cols_per_isplit = (int)(4 * in_steps);
                pl.n_isplit = (int)n_in;
            }
        }
    }
    pl.steps_per_item = pl.o_per_item * (pl.cols_per_isplit / 4);
    if (pl.steps_per_item >= ((int64_t)1 << 30))
        return MTTKRP_ERR_UNSUPPORTED;
    pl.n_splits = pl.n_osplit * pl.n_isplit;
    if (pl.n_splits >= ((int64_t)1 << 30))
        return MTTKRP_ERR_UNSUPPORTED;
    if (k == 0) {
        pl.n_slots = ceil_div(pl.n_splits, pl.group);    // one partial tile per group of wavefronts
        pl.n_items = base_items * pl.n_slots * pl.group;
    } else {
        pl.n_slots = pl.n_splits * pl.n_rowblk;
        pl.n_items = base_items * pl.n_splits;
    }
    if (pl.n_items >= ((int64_t)1 << 31) - 64 || pl.n_slots >= ((int64_t)1 << 31))
        return MTTKRP_ERR_UNSUPPORTED;
    pl.ws_bytes = pl.n_slots > 1
        ? (size_t)pl.n_slots * (size_t)dims[k] * (size_t)R * (size_t)sbytes : 0;
    pl.xcd_remap = tn.xcd_remap == 1;
    pl.wave_cap = (int)tn.waves_per_simd;
    pl.nt_off = tn.nt_loads == 1;
    return MTTKRP_OK;
}

template <typename T, int RB, int JB>
void launch_stream(const StreamArgs<T>& a, dim3 grid, hipStream_t st, int cap, bool nt_off)
{
    // first mode: two wavefront tiles of LDS for the cross-wavefront sum
    size_t lds = a.first_mode && a.group4 ? (size_t)2 * RB * JB * 4 * 64 * sizeof(T) : 0;
    // Resident wavefronts per SIMD can be capped by reserving LDS: a workgroup is one
    // wavefront per SIMD, and a compute unit has 160 KB of LDS.
    if (cap >= 1 && cap <= 7) {
        const size_t want = (size_t)160 * 1024 / (size_t)(cap + 1) + 256;
        if (want <= 65536 && want > lds)
            lds = want;
    }
    // non-temporal tensor loads only when each load instruction reads whole aligned lines
    const bool nt = !nt_off && sizeof(T) == 8 && a.I0 % 16 == 0 && ((uintptr_t)a.X & 127u) == 0;
    if (nt)
        hipLaunchKernelGGL((mttkrp_stream_kernel<T, RB, JB, true>), grid, dim3(kBlockThreads), lds, st, a);
    else
        hipLaunchKernelGGL((mttkrp_stream_kernel<T, RB, JB, false>), grid, dim3(kBlockThreads), lds, st, a);
}

template <typename T, int RB>
void launch_stream_jb(int JB, const StreamArgs<T>& a, dim3 grid, hipStream_t st, int cap, bool nt_off)
{
    switch (JB) {
    case 1: launch_stream<T, RB, 1>(a, grid, st, cap, nt_off); break;
    case 2: launch_stream<T, RB, 2>(a, grid, st, cap, nt_off); break;
    case 3: launch_stream<T, RB, 3>(a, grid, st, cap, nt_off); break;
    default: launch_stream<T, RB, 4>(a, grid, st, cap, nt_off); break;
    }
}

template <typename T>
void launch_stream_rb(int RB, int JB, const StreamArgs<T>& a, dim3 grid, hipStream_t st, int cap, bool nt_off)
{
    switch (RB) {
    case 1: launch_stream_jb<T, 1>(JB, a, grid, st, cap, nt_off); break;
    case 2: launch_stream_jb<T, 2>(JB, a, grid, st, cap, nt_off); break;
    case 3: launch_stream_jb<T, 3>(JB, a, grid, st, cap, nt_off); break;
    default: launch_stream_jb<T, 4>(JB, a, grid, st, cap, nt_off); break;
    }
}

constexpr int kTimingSlots = 512;   // ring of timed calls kept per device

struct TimedCall {
    // before the streaming kernel, between the two kernels, after the combine kernel
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
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
        void* workspace, size_t workspace_bytes, bool own_ws, void* stream,
        const T* lambda = nullptr, double beta = 0.0)
{
    if (!X || !M || !factors)
        return MTTKRP_ERR_INVALID_ARG;
    Plan pl;
    int rc = make_plan(ndim, dims, R, k, (int)sizeof(T), pl);
    if (rc != MTTKRP_OK)
        return rc;
    // Weights and accumulation are applied by the combine kernel, which then always runs.
    const bool scaled = lambda != nullptr || beta != 0.0;
    if (scaled && pl.ws_bytes == 0)
        pl.ws_bytes = (size_t)pl.dims[k] * (size_t)R * sizeof(T);
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
                for (int e = 0; e < 3; ++e)
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
    a.out = pl.ws_bytes > 0 ? ws : M;
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
    a.n_splits = (int32_t)pl.n_splits;
    a.xcd_remap = pl.xcd_remap ? 1 : 0;
    a.group4 = pl.group == kWaves ? 1 : 0;
#ifdef MTTKRP_TRACE
    a.trace = (long long*)(uintptr_t)g_tune.trace_ptr;   // g_mutex is held here
#endif

    int64_t blocks = ceil_div(pl.n_items, kWaves);
    if (a.xcd_remap)
        blocks = ceil_div(blocks, 8) * 8;
    if (blocks >= ((int64_t)1 << 31))
        return MTTKRP_ERR_UNSUPPORTED;

    (void)hipGetLastError();
    if (timing)
        (void)hipEventRecord(tc->ev[0], st);
    launch_stream_rb<T>(pl.RB, pl.JB, a, dim3((unsigned)blocks), st, pl.wave_cap, pl.nt_off);
    if (timing) {
        (void)hipEventRecord(tc->ev[1], st);
        tc->combine = false;
    }
    if (hipGetLastError() != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    if (pl.ws_bytes > 0) {
        const int64_t n_elems = pl.dims[k] * (int64_t)R;
        const int64_t stride_row = k == 0 ? R : pl.n_slots * (int64_t)R;
        const int64_t stride_slot = k == 0 ? pl.dims[0] * (int64_t)R : R;
        hipLaunchKernelGGL((mttkrp_combine_kernel<T>), dim3((unsigned)ceil_div(n_elems, 16)),
                           dim3(256), 0, st, (const T*)ws, M, n_elems, R, (int)pl.n_slots,
                           stride_row, stride_slot, lambda, beta);
        if (timing) {
            (void)hipEventRecord(tc->ev[2], st);
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

size_t mttkrp_dense_ex_workspace_bytes(int ndim, const int64_t* dims, int R, int k, int dtype_bytes)
{
    Plan pl;
    if (make_plan(ndim, dims, R, k, dtype_bytes, pl) != MTTKRP_OK)
        return (size_t)-1;
    return pl.ws_bytes > 0 ? pl.ws_bytes : (size_t)pl.dims[k] * (size_t)R * (size_t)dtype_bytes;
}

int mttkrp_dense_f64_ex(int ndim, const int64_t* dims, const double* X,
                        const double* const* factors, int R, int k, const double* lambda,
                        double beta, double* M, void* workspace, size_t workspace_bytes,
                        void* stream)
{
    return run<double>(ndim, dims, X, factors, R, k, M, workspace, workspace_bytes,
                       workspace == nullptr, stream, lambda, beta);
}

int mttkrp_dense_f32_ex(int ndim, const int64_t* dims, const float* X, const float* const* factors,
                        int R, int k, const float* lambda, float beta, float* M, void* workspace,
                        size_t workspace_bytes, void* stream)
{
    return run<float>(ndim, dims, X, factors, R, k, M, workspace, workspace_bytes,
                      workspace == nullptr, stream, lambda, (double)beta);
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
                for (int e = 0; e < 3; ++e)
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
    if (hipEventSynchronize(tc.combine ? tc.ev[2] : tc.ev[1]) != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    if (hipEventElapsedTime(stream_ms, tc.ev[0], tc.ev[1]) != hipSuccess)
        return MTTKRP_ERR_DEVICE;
    if (tc.combine && hipEventElapsedTime(combine_ms, tc.ev[1], tc.ev[2]) != hipSuccess)
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
    } else if (!strcmp(key, "max_col_blocks")) {
        if (value > 4) return MTTKRP_ERR_INVALID_ARG;
        g_tune.max_col_blocks = value;
    } else if (!strcmp(key, "first_group")) {
        if (value != 0 && value != 1 && value != 4) return MTTKRP_ERR_INVALID_ARG;
        g_tune.first_group = value;
    } else if (!strcmp(key, "waves_per_simd")) {
        if (value > 8) return MTTKRP_ERR_INVALID_ARG;
        g_tune.waves_per_simd = value;
#ifdef MTTKRP_TRACE
    } else if (!strcmp(key, "trace_ptr")) {
        g_tune.trace_ptr = value;
#endif
    } else if (!strcmp(key, "nt_loads")) {
        if (value > 1) return MTTKRP_ERR_INVALID_ARG;
        g_tune.nt_loads = value;
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
