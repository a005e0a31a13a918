// Dense projection Z = X W on the matrix cores (fp32 MFMA, fp32 accumulate): the contraction
// inside GCNConv and the GAT layer (layers named in the paper, section 3).  X is tall and
// skinny ([rows x k], k ~ 100), W is small ([k x n], n <= a few hundred).
//
// A wavefront owns 32 rows and BN/32 accumulator tiles of v_mfma_f32_32x32x2_f32.  X fragments go from global
// memory straight to registers, 64 k-values ("sub-slab") at a time: the lane (r = lane % 32, half = lane / 32)
// reads the 32 consecutive floats X[row0 + r][k0 + 32*half ..] -- one full 128-byte line per lane,
// eight 128-bit loads issued back to back -- and feeds value j of its s-th group of four to MFMA
// (s, j), whose B operand is W[k0 + 32*half + 4*s + j][col].  The k order inside a sub-slab is thus
// permuted identically for both operands, which leaves the sum unchanged.
// W sits in LDS transposed ([col][k], k contiguous) so that the four B values of a group come from
// one 128-bit LDS read; the 16-byte groups of a column are xor-swizzled with (col % 8) so that the
// lanes of a read (same group, consecutive columns) fall into different banks without padding.
//
// Fast kernel (k <= 128, k and n multiples of 4): one block of twelve wavefronts per compute unit stages its
// columns of W once, then every wavefront walks over 32-row tiles.
// General kernel (any shape, ragged edges): one 128-row tile per block of four wavefronts, W re-staged per 64-k slab.
//
// What the direct global-to-register path costs (timestamps taken inside the fast kernel at the GCN size): the
// address unit takes a 128-bit load whose lanes lie in different rows at about one lane per cycle, so issuing the
// sixteen loads of a tile for twelve wavefronts keeps a compute unit busy for 8-9 us before the first MFMA --
// whether the two halves of a wavefront share lines or not (both layouts were measured).
#include "gnn_internal.h"

#include <algorithm>

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kFastWavesMax = 8, kFastThreadsMax = 64 * kFastWavesMax;   // fast kernel: one block per compute unit
constexpr int kLdsBytes = 160 * 1024;
constexpr int kRowsPerWave = 32;
constexpr int kRowsPerBlock = 4 * kRowsPerWave;
constexpr int kSlab = 64;             // k-values per X register buffer / per staged W slab in the fallback

// What the store does after the product: optional per-row scale, per-column bias, relu (in that order).
struct XwEpilogue {
    const float *row_scale = nullptr;
    const float *bias = nullptr;
    int relu = 0;
    gnn_column_norm norm;   // applied to X on the way in when norm.mean is set (fast kernel only)
    int w_transposed = 0;   // w is stored [n x k]: the product is X w^T (fast kernel only)
};

struct AFrag {
    float v[8][4];
};

// Loads are unconditional (no branches, so that the hardware load counter can be waited on
// precisely and the next buffer's loads stay in flight): rows past the end are clamped to the last
// row (their results are never stored) and k positions past the end are clamped into the row (their
// values meet zero-filled rows of W in LDS, and inputs are finite by contract).
// KSTEPS (even, <= 8) = groups of four k-values a lane reads: a sub-slab then spans 8 * KSTEPS k-values, the
// lower half of the wavefront taking the first 4 * KSTEPS of them (narrow inputs do a fraction of the MFMA work).
template <bool VEC4, int KSTEPS = 8>
__device__ __forceinline__ void load_a(AFrag &a, const float *__restrict__ x, int64_t rows, int k, int64_t row,
                                       int k0, int half)
{
    const float *xrow = x + min(row, rows - 1) * (int64_t)k;
#pragma unroll
    for (int s = 0; s < KSTEPS; ++s) {
        const int kb = k0 + 4 * KSTEPS * half + 4 * s;
        if constexpr (VEC4) {
            const float4 t = *reinterpret_cast<const float4 *>(xrow + min(kb, k - 4));   // k % 4 == 0
            a.v[s][0] = t.x; a.v[s][1] = t.y; a.v[s][2] = t.z; a.v[s][3] = t.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) a.v[s][j] = xrow[min(kb + j, k - 1)];
        }
    }
}

// LDS position of W[k][col] for a column block stored as [col][kp] floats, kp a multiple of 32.
// The 16-byte chunk index is xor-ed with a function of the column so that the 128-bit reads of the MFMA operand
// (lane = column, every lane the same chunk) are free of bank conflicts.  On this part a 128-bit LDS read is served
// 16 lanes per cycle over 64 banks, and the 16 lanes are not neighbours: lanes {0-3, 12-15, 20-23, 24-27} share a
// cycle, so do {4-7, 8-11, 16-19, 28-31}, and the same with 32 added (measured with two active lanes and the bank
// conflict counter).  A column is kp / 4 chunks long: when that is a multiple of 16 the column's start does not
// move the bank and the low four bits of the column separate the 16 lanes of a cycle; otherwise columns alternate
// between the two halves of the banks and bits 1-3 of the column separate the eight even and the eight odd ones.
__device__ __forceinline__ int w_lds_index(int col, int k, int kp)
{
    const int swizzle = (kp & 32) ? ((col >> 1) & 7) : (col & 15);
    return col * kp + ((((k >> 2) ^ swizzle) << 2) | (k & 3));
}

// Swizzle of the per-wavefront X / output slab: chunk c of row r (32 rows of eight 16-byte chunks) lies at slot
// 8 r + (c ^ slab_swizzle(r)).  Chosen so that all four ways the slab is touched are free of bank conflicts:
// 128-bit reads with lane = row (MFMA operand; cycle groups as above, 64 banks), 128-bit reads with eight
// neighbouring lanes = one row (staged output), 128-bit writes with eight neighbouring lanes = one row (tile) and
// with lane = row (accumulators) -- writes are served eight neighbouring lanes per cycle over 32 banks.
__device__ __forceinline__ int slab_swizzle(int r)
{
    return ((r >> 1) & 3) | (((r ^ (r >> 3)) & 1) << 2);
}

// acc += (A(sub-slab) * W(sub-slab))^T: the W fragment is fed as the MFMA's first operand and the X
// fragment as its second, so the 32x32 accumulator tile holds Z transposed -- register v of lane l is
// Z[row0 + l%32][col0 + 8*(v/4) + 4*(l/32) + v%4] -- and a lane's four consecutive registers are four
// consecutive columns of one output row (one 128-bit store).  kbase = first k of this lane's half of the sub-slab relative to
// the staged block (a multiple of 32); r = lane % 32.  Always the full 64 k-values, straight-line
// code (k positions past the end of the matrix multiply zero-filled W rows).
template <int NT>
__device__ __forceinline__ void load_b(float4 (&b)[NT], const float *ws, int kp, int k4, int r)
{
#pragma unroll
    for (int t = 0; t < NT; ++t) b[t] = *reinterpret_cast<const float4 *>(ws + w_lds_index(t * 32 + r, k4, kp));
}

template <int NT>
__device__ __forceinline__ void mfma_step(floatx16 (&acc)[NT], const float (&a)[4], const float4 (&b)[NT])
{
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[t].x, a[0], acc[t], 0, 0, 0);
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[t].y, a[1], acc[t], 0, 0, 0);
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[t].z, a[2], acc[t], 0, 0, 0);
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[t].w, a[3], acc[t], 0, 0, 0);
}

template <int NT, int KSTEPS = 8>
__device__ __forceinline__ void mfma_subslab(floatx16 (&acc)[NT], const AFrag &a, const float *ws, int kp, int kbase,
                                             int r)
{
    // W fragments are read one step ahead of the MFMAs that use them; the scheduling barriers keep
    // the compiler from hoisting all the steps' reads (which would cost occupancy).
    static_assert(KSTEPS % 2 == 0 && KSTEPS <= 8, "steps come in pairs");
    float4 b0[NT], b1[NT];
    load_b<NT>(b0, ws, kp, kbase, r);
#pragma unroll
    for (int s = 0; s < KSTEPS; s += 2) {
        load_b<NT>(b1, ws, kp, kbase + 4 * (s + 1), r);
        mfma_step<NT>(acc, a.v[s], b0);
        __builtin_amdgcn_sched_barrier(0);
        if (s + 2 < KSTEPS) load_b<NT>(b0, ws, kp, kbase + 4 * (s + 2), r);
        mfma_step<NT>(acc, a.v[s + 1], b1);
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Guarded store of the (transposed) accumulator tiles, for ragged edges.  Epilogue: optional per-row scale,
// then optional per-column bias, then optional relu.
template <int NT>
__device__ __forceinline__ void store_tile(const floatx16 (&acc)[NT], int64_t row0, int64_t rows, int n0, int n,
                                           int r, int half, const float *__restrict__ row_scale,
                                           const float *__restrict__ bias, int relu, float *__restrict__ z)
{
    const int64_t row = row0 + r;
    if (row >= rows) return;
    const float sc = row_scale ? row_scale[row] : 1.0f;
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int col = n0 + t * 32 + 8 * (v / 4) + 4 * half + (v % 4);
            if (col < n) {
                float o = acc[t][v] * sc;
                if (bias) o += bias[col];
                if (relu) o = fmaxf(o, 0.0f);
                z[row * n + col] = o;
            }
        }
}

// Stages W[k0 .. k0+KK) x [n0 .. n0+BN) into LDS, transposed and swizzled (zero-filled outside the matrix).
// KK is a multiple of 32 and is the LDS row length.  vec4 = n % 4 == 0 and w is 16-byte aligned: a group of four
// columns is inside or outside the matrix as a whole.  All of a thread's loads are issued before the first LDS
// write (addresses outside the matrix are replaced by the matrix's first group, values by zero: no branches
// between the loads, so one round trip to memory instead of one per pass).
template <int BN, int KK, int NTHREADS>
struct WStage {
    static constexpr int G = BN / 4, TOTAL = KK * G, ITERS = (TOTAL + NTHREADS - 1) / NTHREADS;
    static_assert(KK % 16 == 0 && G % 4 == 0, "staging blocks of 16 k-values x 4 column groups");
    float4 v[ITERS];

    // Which 128-bit group (row kk of W, four columns from c) a staging index stands for.  64 consecutive
    // indices -- a wavefront -- cover 16 consecutive rows x 4 neighbouring column groups: the global reads come in
    // 64-byte pieces, and the four transposed LDS writes of a pass spread over all banks (16 k-values of a column
    // are 16 consecutive words; the neighbouring column groups land in other bank groups through the swizzle),
    // where one row x 64 column groups would put every lane of a write into the same bank.
    static __device__ __forceinline__ void decode(int idx, int &kk, int &c)
    {
        constexpr int KBLOCKS = KK / 16;
        const int blk = idx >> 6, l = idx & 63;
        kk = (blk % KBLOCKS) * 16 + (l & 15);
        c = ((blk / KBLOCKS) * 4 + (l >> 4)) * 4;
    }

    // transposed: w is stored [n x k] (the product is X w^T); the four columns of a group are then four rows of
    // the array, read as single words -- lanes with neighbouring k still read neighbouring addresses.
    __device__ __forceinline__ void load(const float *__restrict__ w, int k, int n, int k0, int n0, bool transposed = false)
    {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int idx = min((int)threadIdx.x + it * NTHREADS, TOTAL - 1);   // a last, partial pass loads something valid
            int kk, c;
            decode(idx, kk, c);
            const bool inside = k0 + kk < k && n0 + c < n;
            if (transposed) {   // the same for every thread of the launch
                const float *p = inside ? w + (int64_t)(n0 + c) * k + k0 + kk : w;
                const int64_t step = inside ? k : 0;
                v[it] = make_float4(p[0], p[step], p[2 * step], p[3 * step]);
            } else {
                const float *p = inside ? w + (int64_t)(k0 + kk) * n + n0 + c : w;
                v[it] = *reinterpret_cast<const float4 *>(p);
            }
        }
    }

    __device__ __forceinline__ void store(float *ws, int k, int n, int k0, int n0) const
    {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int idx = threadIdx.x + it * NTHREADS;
            int kk, c;
            decode(min(idx, TOTAL - 1), kk, c);
            const bool inside = k0 + kk < k && n0 + c < n;
            if (idx < TOTAL) {
                ws[w_lds_index(c + 0, kk, KK)] = inside ? v[it].x : 0.0f;
                ws[w_lds_index(c + 1, kk, KK)] = inside ? v[it].y : 0.0f;
                ws[w_lds_index(c + 2, kk, KK)] = inside ? v[it].z : 0.0f;
                ws[w_lds_index(c + 3, kk, KK)] = inside ? v[it].w : 0.0f;
            }
        }
    }
};

template <int BN, int KK, int NTHREADS>
__device__ __forceinline__ void stage_w(float *ws, const float *__restrict__ w, int k, int n, int k0, int n0, bool vec4)
{
    if (vec4) {
        WStage<BN, KK, NTHREADS> st;
        st.load(w, k, n, k0, n0);
        st.store(ws, k, n, k0, n0);
    } else {
        constexpr int TOTAL = KK * BN;
#pragma unroll 8
        for (int idx = threadIdx.x; idx < TOTAL; idx += NTHREADS) {
            const int kk = idx / BN, c = idx - kk * BN;
            float v = 0.0f;
            if (k0 + kk < k && n0 + c < n) v = w[(int64_t)(k0 + kk) * n + n0 + c];
            ws[w_lds_index(c, kk, KK)] = v;
        }
    }
}

// Fast path: k <= 128, k and n multiples of 4, 16-byte aligned rows.  One block of up to eight wavefronts per
// compute unit (two per SIMD) stages its columns of W once -- one copy in LDS serves all of them -- and then every
// wavefront walks over 32-row tiles on its own, with no barrier after the first.
//
// X reaches the matrix cores through a per-wavefront LDS slab that holds one tile (32 rows x 32 KQ k-values, 4 KB
// per quarter of 32 k-values).  Global loads are coalesced: in each of a quarter's four load instructions eight
// neighbouring lanes read one row's 128-byte segment, so an instruction touches eight full-width segments instead
// of 64 different lines (the address unit handles a 128-bit load whose lanes all lie in different rows at about
// one lane per cycle: the loads of a tile then take microseconds just to issue).  The lanes write their 16-byte
// chunks to the slab, chunk c of row r of a quarter at slot 8 r + (c ^ slab_swizzle(r)), and read them back in the MFMA
// operand layout (lane = row, two k-halves): neither direction has a bank conflict (see slab_swizzle).  LDS
// operations of one wavefront execute in order, so the slab needs no barrier and no second copy.
// A whole tile is in flight per wavefront: as soon as a tile's registers have been written to the slab, all loads
// of the wavefront's next tile are issued back to back (rows that are not a multiple of 128 bytes share lines
// between quarters; requested together, such a line is fetched once), and they have the whole tile's MFMAs to
// arrive.  The accumulators of all NT column tiles stay live (k is the outer loop), so X is read once per row
// whatever the output width.
//
// k order: in quarter q, step s (of S) and lane half h, MFMA j consumes k = 32 q + 4 (h S + s) + j from both
// operands; S = 4 except in the last quarter, where it is just large enough for the k-values that exist (no MFMA
// work on padding beyond that: k = 100 runs 3 x 16 + 2 k-steps instead of 64).
constexpr int kSlabFloats = 32 * 32;    // one quarter of a tile

typedef float v4f __attribute__((ext_vector_type(4)));

struct QuarterRegs {
    v4f v0, v1, v2, v3;
};

// The quarters of one tile as named members (indexed at compile time only).
struct TileRegs {
    QuarterRegs q0, q1, q2, q3;
    template <int Q>
    __device__ __forceinline__ QuarterRegs &quarter()
    {
        if constexpr (Q == 0) return q0;
        else if constexpr (Q == 1) return q1;
        else if constexpr (Q == 2) return q2;
        else return q3;
    }
};

template <int KQ, int Q = 0>
__device__ __forceinline__ void load_tile(TileRegs &t, const float *__restrict__ x, int64_t rows, int k, int64_t row0,
                                          int lane);
template <int KQ, int Q = 0>
__device__ __forceinline__ void write_tile(float *slab, TileRegs &t, int lane);

// The four coalesced loads of quarter q of the tile starting at row0: instruction i covers rows 8 i .. 8 i + 7,
// lane l the chunk l % 8 of row 8 i + l / 8.  Unconditional (clamped) addresses: rows past the end read the last
// row (never stored), chunks past the end of a row read the row's last chunk (they meet zero rows of W).
__device__ __forceinline__ void load_quarter(QuarterRegs &t, const float *__restrict__ x, int64_t rows, int k,
                                             int64_t row0, int q, int lane)
{
    const int kb = min(32 * q + 4 * (lane & 7), k - 4);
    const int64_t r0 = row0 + (lane >> 3);
    t.v0 = *reinterpret_cast<const v4f *>(x + min(r0, rows - 1) * (int64_t)k + kb);
    t.v1 = *reinterpret_cast<const v4f *>(x + min(r0 + 8, rows - 1) * (int64_t)k + kb);
    t.v2 = *reinterpret_cast<const v4f *>(x + min(r0 + 16, rows - 1) * (int64_t)k + kb);
    t.v3 = *reinterpret_cast<const v4f *>(x + min(r0 + 24, rows - 1) * (int64_t)k + kb);
}

// Chunk c of row r goes to slot 8 r + (c ^ slab_swizzle(r)); the lane's rows are lane / 8 + 8 i, whose swizzles
// differ in bit 2 for odd i.
__device__ __forceinline__ void write_quarter(float *slab, const QuarterRegs &t, int lane)
{
    const int r = lane >> 3;
    const int c0 = (lane & 7) ^ slab_swizzle(r), c1 = c0 ^ 4;
    float *p = slab + 4 * 8 * r;
    *reinterpret_cast<v4f *>(p + 4 * c0) = t.v0;
    *reinterpret_cast<v4f *>(p + 4 * (64 + c1)) = t.v1;
    *reinterpret_cast<v4f *>(p + 4 * (128 + c0)) = t.v2;
    *reinterpret_cast<v4f *>(p + 4 * (192 + c1)) = t.v3;
}

// The column normalisation of the four k-values a lane holds of every row of a quarter (the lane's chunk is the
// same in all four loads of a quarter): mean, 1/sqrt(var + eps), gamma, beta per value.
struct NormQuarter {
    v4f mean, inv, gamma, beta;
};

struct NormRegs {
    NormQuarter q0, q1, q2, q3;
    template <int Q>
    __device__ __forceinline__ NormQuarter &quarter()
    {
        if constexpr (Q == 0) return q0;
        else if constexpr (Q == 1) return q1;
        else if constexpr (Q == 2) return q2;
        else return q3;
    }
};

template <int KQ, int Q = 0>
__device__ __forceinline__ void load_norm(NormRegs &nr, const gnn_column_norm &cn, int k, int lane)
{
    if constexpr (Q < KQ) {
        const int kb = min(32 * Q + 4 * (lane & 7), k - 4);   // the chunk load_quarter reads
        NormQuarter &nq = nr.quarter<Q>();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            nq.mean[c] = cn.mean[kb + c];
            nq.inv[c] = 1.0f / sqrtf(cn.var[kb + c] + cn.eps);
            nq.gamma[c] = cn.gamma ? cn.gamma[kb + c] : 1.0f;
            nq.beta[c] = cn.beta ? cn.beta[kb + c] : 0.0f;
        }
        load_norm<KQ, Q + 1>(nr, cn, k, lane);
    }
}

__device__ __forceinline__ v4f norm_chunk(v4f x, const NormQuarter &nq, int relu)
{
    v4f y;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        float v = nq.gamma[c] * ((x[c] - nq.mean[c]) * nq.inv[c]) + nq.beta[c];
        y[c] = relu ? fmaxf(v, 0.0f) : v;
    }
    return y;
}

template <int KQ, int Q = 0>
__device__ __forceinline__ void norm_tile(TileRegs &t, NormRegs &nr, int relu)
{
    if constexpr (Q < KQ) {
        QuarterRegs &qr = t.quarter<Q>();
        const NormQuarter &nq = nr.quarter<Q>();
        qr.v0 = norm_chunk(qr.v0, nq, relu);
        qr.v1 = norm_chunk(qr.v1, nq, relu);
        qr.v2 = norm_chunk(qr.v2, nq, relu);
        qr.v3 = norm_chunk(qr.v3, nq, relu);
        norm_tile<KQ, Q + 1>(t, nr, relu);
    }
}

template <int KQ, int Q>
__device__ __forceinline__ void load_tile(TileRegs &t, const float *__restrict__ x, int64_t rows, int k, int64_t row0,
                                          int lane)
{
    if constexpr (Q < KQ) {
        load_quarter(t.quarter<Q>(), x, rows, k, row0, Q, lane);
        load_tile<KQ, Q + 1>(t, x, rows, k, row0, lane);
    }
}

template <int KQ, int Q>
__device__ __forceinline__ void write_tile(float *slab, TileRegs &t, int lane)
{
    if constexpr (Q < KQ) {
        write_quarter(slab + Q * kSlabFloats, t.quarter<Q>(), lane);
        write_tile<KQ, Q + 1>(slab, t, lane);
    }
}

// The operands of one step of four k-values for all NT column tiles: X chunk `chunk` of the lane's row from the
// slab, W[32 q + 4 chunk ..][column tiles] from the staged block.
template <int NT>
struct StepOperands {
    float4 a;
    float4 b[NT];
    __device__ __forceinline__ void load(const float *slab, const float *ws, int kp, int q, int chunk, int r)
    {
        a = *reinterpret_cast<const float4 *>(slab + 4 * (8 * r + (chunk ^ slab_swizzle(r))));
        load_b<NT>(b, ws, kp, 32 * q + 4 * chunk, r);
    }
};

// W fragment as the MFMA's first operand, X fragment as its second, so that the accumulator holds the tile
// transposed (see the store).
template <int NT>
__device__ __forceinline__ void step_mfmas(floatx16 (&acc)[NT], const StepOperands<NT> &o)
{
    const float av[4] = {o.a.x, o.a.y, o.a.z, o.a.w};
    mfma_step<NT>(acc, av, o.b);
}

// The four steps of a full quarter, operands read from LDS one step ahead of the MFMAs that use them (the
// scheduling barriers keep the compiler from hoisting all reads to the front, which would cost registers).
template <int NT>
__device__ __forceinline__ void full_quarter(floatx16 (&acc)[NT], const float *slab, const float *ws, int kp, int q,
                                             int half, int r)
{
    StepOperands<NT> o0, o1;
    o0.load(slab, ws, kp, q, 4 * half, r);
    o1.load(slab, ws, kp, q, 4 * half + 1, r);
    step_mfmas<NT>(acc, o0);
    __builtin_amdgcn_sched_barrier(0);
    o0.load(slab, ws, kp, q, 4 * half + 2, r);
    step_mfmas<NT>(acc, o1);
    __builtin_amdgcn_sched_barrier(0);
    o1.load(slab, ws, kp, q, 4 * half + 3, r);
    step_mfmas<NT>(acc, o0);
    __builtin_amdgcn_sched_barrier(0);
    step_mfmas<NT>(acc, o1);
}

// A finished tile on its way to memory.  The accumulator holds it transposed: register v of lane l is
// Z[row0 + l % 32][8 (v / 4) + 4 (l / 32) + v % 4] of its column tile, i.e. a lane owns 16-byte pieces of one row that
// lie 32 bytes apart -- stored like that, every store instruction would touch 32 different lines with 32 bytes
// each.  The tile goes through the wavefront's LDS slab instead, one 32 x 32 column tile at a time, and comes back
// in the layout of the quarter loads (eight neighbouring lanes = one row's 128 bytes): a store instruction then
// writes eight full 128-byte segments.
template <int NT>
struct OutRegs {
    v4f v[NT][4];   // [column tile][i]: columns 4 (lane % 8) .. + 3 of row lane / 8 + 8 i
};

template <int NT>
__device__ __forceinline__ void stage_tile(OutRegs<NT> &o, const floatx16 (&acc)[NT], float *slab, int lane)
{
    const int r = lane & 31, half = lane >> 5;
    const int rr = lane >> 3;
    const int rc0 = (lane & 7) ^ slab_swizzle(rr), rc1 = rc0 ^ 4;   // rows rr + 8 i: bit 2 flips for odd i
    const float *rp = slab + 4 * 8 * rr;
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const v4f t = {acc[tt][4 * g], acc[tt][4 * g + 1], acc[tt][4 * g + 2], acc[tt][4 * g + 3]};
            *reinterpret_cast<v4f *>(slab + 4 * (8 * r + ((2 * g + half) ^ slab_swizzle(r)))) = t;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) o.v[tt][i] = *reinterpret_cast<const v4f *>(rp + 4 * (64 * i + ((i & 1) ? rc1 : rc0)));
    }
}

// Epilogue (row scale, bias, relu, in that order) and the stores of a staged tile starting at row0.
// The row factors of the four rows a lane stores in a tile (clamped rows past the end: never stored).
struct RowScales {
    float s[4];
};

__device__ __forceinline__ void load_row_scales(RowScales &rs, const float *__restrict__ row_scale, int64_t row0,
                                                int64_t rows, int lane)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) rs.s[i] = row_scale[min(row0 + (lane >> 3) + 8 * i, rows - 1)];
}

template <int NT, bool SCALED>
__device__ __forceinline__ void store_staged_tile(const OutRegs<NT> &o, const RowScales &rs, int64_t row0, int64_t rows,
                                                  int n, int n0, int lane, const float *__restrict__ bias, int relu,
                                                  float *__restrict__ z)
{
    const int c4 = 4 * (lane & 7);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t row = row0 + (lane >> 3) + 8 * i;
        if (row >= rows) continue;   // rows past the end in a ragged last tile
        float sc = 1.0f;
        if constexpr (SCALED) sc = rs.s[i];
#pragma unroll
        for (int tt = 0; tt < NT; ++tt) {
            const int col = n0 + 32 * tt + c4;
            if (col >= n) continue;   // n % 4 == 0: a group of four columns is inside or outside as a whole
            v4f v = o.v[tt][i] * sc;
            if (bias) {
                const v4f b = *reinterpret_cast<const v4f *>(bias + col);
                v += b;
            }
            if (relu) v = {fmaxf(v.x, 0.0f), fmaxf(v.y, 0.0f), fmaxf(v.z, 0.0f), fmaxf(v.w, 0.0f)};
            *reinterpret_cast<v4f *>(z + row * n + col) = v;
        }
    }
}

// Wavefronts per block: as many as the LDS holds slabs for next to the staged W, at most eight.
template <int NT, int KQ>
constexpr int fast_waves()
{
    const int fit = (kLdsBytes - NT * 32 * KQ * 32 * 4) / (KQ * kSlabFloats * 4);
    return fit < kFastWavesMax ? fit : kFastWavesMax;
}

template <int NT, int KQ, bool SCALED, bool NORM = false>
__global__ __launch_bounds__(kFastThreadsMax) void xw_fast_kernel(const float *__restrict__ x, int k,
                                                                  const float *__restrict__ w, int n,
                                                                  const float *__restrict__ row_scale,
                                                                  const float *__restrict__ bias, int relu,
                                                                  float *__restrict__ z, int64_t rows,
                                                                  const gnn_column_norm cn, int w_transposed)
{
    constexpr int BN = NT * 32;
    constexpr int KP = KQ * 32;
    constexpr int WAVES = fast_waves<NT, KQ>();
    constexpr int THREADS = 64 * WAVES;
    // W is staged by the first kStageThreads threads (whole wavefronts), all of a thread's loads going out at once.
    constexpr int kStageThreads = (KP * BN / 4) < THREADS ? (KP * BN / 4) : THREADS;
    static_assert(kStageThreads % 64 == 0 && WAVES >= 2, "staging threads");
    extern __shared__ __align__(16) float lds[];   // [BN][KP] of W, swizzled; then one slab per wavefront
    float *ws = lds;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float *slab = lds + BN * KP + wave * (KQ * kSlabFloats);
    const int r = lane & 31, half = lane >> 5;
    const int n0 = blockIdx.y * BN;
    const int64_t num_tiles = (rows + kRowsPerWave - 1) / kRowsPerWave;
    // steps of the last quarter: its k-values, in chunks of four, split over the two lane halves
    const int last_chunks = (k - 32 * (KQ - 1) + 3) / 4;
    const int last_steps = (last_chunks + 1) / 2;

    // Tile numbers go round the blocks first, then round the wavefronts of a block, so that a last, partly
    // filled round puts one tile on as many compute units as possible.
    const int64_t stride = (int64_t)gridDim.x * WAVES;
    int64_t tile = (int64_t)wave * gridDim.x + blockIdx.x;

    // W's loads are issued first, then the first tile's (clamped addresses: safe also for a wavefront without a
    // tile), which stay in flight while W is written to LDS.
    TileRegs t;
    NormRegs nr;
    if constexpr (NORM) load_norm<KQ>(nr, cn, k, lane);
    RowScales rs_next{}, rs_this{}, rs_prev{};   // row factors travel with their tile: loaded with it, used at its store
    {
        WStage<BN, KP, kStageThreads> st;
        const bool stager = threadIdx.x < kStageThreads;   // whole wavefronts
        if (stager) st.load(w, k, n, 0, n0, w_transposed != 0);
        __builtin_amdgcn_sched_barrier(0);
        load_tile<KQ>(t, x, rows, k, tile * kRowsPerWave, lane);
        if constexpr (SCALED) load_row_scales(rs_next, row_scale, tile * kRowsPerWave, rows, lane);
        __builtin_amdgcn_sched_barrier(0);
        if (stager) st.store(ws, k, n, 0, n0);
    }
    __syncthreads();

    // The stores of a tile are issued inside the next tile, after its slab writes: the memory counter is waited on
    // in order, so a wait for loads that were issued before the stores would otherwise wait for the stores as well.
    floatx16 acc[NT];
    OutRegs<NT> out;
    int64_t prev_row0 = -1;   // first row of the tile whose staged results `out` still holds
    for (; tile < num_tiles; tile += stride) {
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (NORM) norm_tile<KQ>(t, nr, cn.relu);   // k-values past the row's end meet zero rows of W
        write_tile<KQ>(slab, t, lane);
        __builtin_amdgcn_sched_barrier(0);   // the next tile is loaded into the same registers: no copies
        if (prev_row0 >= 0) store_staged_tile<NT, SCALED>(out, rs_prev, prev_row0, rows, n, n0, lane, bias, relu, z);
#pragma unroll
        for (int tt = 0; tt < NT; ++tt)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tt][v] = 0.0f;
        __builtin_amdgcn_sched_barrier(0);
        rs_this = rs_next;   // arrived with this tile's X (waited for by the slab writes above)
        load_tile<KQ>(t, x, rows, k, (tile + stride) * kRowsPerWave, lane);
        if constexpr (SCALED) load_row_scales(rs_next, row_scale, (tile + stride) * kRowsPerWave, rows, lane);
        __builtin_amdgcn_sched_barrier(0);   // the loads go out here, not where the compiler would sink them to
#pragma unroll
        for (int q = 0; q + 1 < KQ; ++q) full_quarter<NT>(acc, slab + q * kSlabFloats, ws, KP, q, half, r);
        for (int s = 0; s < last_steps; ++s) {
            StepOperands<NT> o;
            o.load(slab + (KQ - 1) * kSlabFloats, ws, KP, KQ - 1, last_steps * half + s, r);
            step_mfmas<NT>(acc, o);
        }
        __builtin_amdgcn_sched_barrier(0);
        stage_tile<NT>(out, acc, slab, lane);   // LDS operations of a wavefront run in order: the slab's X data has been read
        rs_prev = rs_this;
        prev_row0 = tile * kRowsPerWave;
    }
    __builtin_amdgcn_sched_barrier(0);
    if (prev_row0 >= 0) store_staged_tile<NT, SCALED>(out, rs_prev, prev_row0, rows, n, n0, lane, bias, relu, z);
}

template <int NT, bool VEC4>
__global__ __launch_bounds__(kThreads) void xw_slab_kernel(const float *__restrict__ x, int64_t rows, int k,
                                                           const float *__restrict__ w, int n,
                                                           const float *__restrict__ row_scale,
                                                           const float *__restrict__ bias, int relu,
                                                           float *__restrict__ z, int w_vec4, int64_t first_row_tile)
{
    constexpr int BN = NT * 32;
    __shared__ __align__(16) float ws[kSlab * BN];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, half = lane >> 5;
    const int64_t row0 = (first_row_tile + blockIdx.x) * kRowsPerBlock + wave * kRowsPerWave;
    const int n0 = blockIdx.y * BN;

    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    for (int k0 = 0; k0 < k; k0 += kSlab) {
        AFrag a;
        load_a<VEC4>(a, x, rows, k, row0 + r, k0, half);
        __syncthreads();
        stage_w<BN, kSlab, kThreads>(ws, w, k, n, k0, n0, w_vec4 != 0);
        __syncthreads();
        mfma_subslab<NT>(acc, a, ws, kSlab, 32 * half, r);
    }
    store_tile<NT>(acc, row0, rows, n0, n, r, half, row_scale, bias, relu, z);
}

int device_cu_count()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
            cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

template <int NT>
gnn_status launch_general(const float *d_x, int64_t rows, int k, const float *d_w, int n, const XwEpilogue &ep,
                          float *d_z, bool x_vec4, bool w_vec4, int64_t first_row_tile, hipStream_t s)
{
    const int64_t row_tiles = gnn_div_up(rows, kRowsPerBlock) - first_row_tile;
    if (row_tiles <= 0) return GNN_OK;
    const dim3 grid((unsigned)row_tiles, (unsigned)gnn_div_up(n, NT * 32));
    if (x_vec4)
        hipLaunchKernelGGL((xw_slab_kernel<NT, true>), grid, dim3(kThreads), 0, s, d_x, rows, k, d_w, n, ep.row_scale,
                           ep.bias, ep.relu, d_z, w_vec4 ? 1 : 0, first_row_tile);
    else
        hipLaunchKernelGGL((xw_slab_kernel<NT, false>), grid, dim3(kThreads), 0, s, d_x, rows, k, d_w, n, ep.row_scale,
                           ep.bias, ep.relu, d_z, w_vec4 ? 1 : 0, first_row_tile);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

template <int NT, int KQ>
gnn_status launch_fast(const float *d_x, int64_t rows, int k, const float *d_w, int n, const XwEpilogue &ep,
                       float *d_z, hipStream_t s)
{
    constexpr int BN = NT * 32;   // output columns per block
    constexpr int WAVES = fast_waves<NT, KQ>();
    const int64_t tiles = gnn_div_up(rows, kRowsPerWave);
    const size_t lds = ((size_t)KQ * 32 * BN + (size_t)WAVES * KQ * kSlabFloats) * sizeof(float);
    // One resident block per compute unit (fewer where there are several column blocks or few rows: then at
    // least one tile per block, so that small inputs still spread over the chip).
    const int col_blocks = (int)gnn_div_up(n, BN);
    const int64_t blocks = std::max<int64_t>(1, std::min<int64_t>(device_cu_count() / col_blocks, tiles));
    const dim3 grid((unsigned)blocks, (unsigned)col_blocks);
    if (ep.norm.mean) {   // the one user: a graph convolution (row factors) reading batch-normalised rows
        if (!ep.row_scale) return GNN_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((xw_fast_kernel<NT, KQ, true, true>), grid, dim3(64 * WAVES), lds, s, d_x, k, d_w, n,
                           ep.row_scale, ep.bias, ep.relu, d_z, rows, ep.norm, ep.w_transposed);
    } else if (ep.row_scale)
        hipLaunchKernelGGL((xw_fast_kernel<NT, KQ, true>), grid, dim3(64 * WAVES), lds, s, d_x, k, d_w, n,
                           ep.row_scale, ep.bias, ep.relu, d_z, rows, ep.norm, ep.w_transposed);
    else
        hipLaunchKernelGGL((xw_fast_kernel<NT, KQ, false>), grid, dim3(64 * WAVES), lds, s, d_x, k, d_w, n,
                           ep.row_scale, ep.bias, ep.relu, d_z, rows, ep.norm, ep.w_transposed);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

template <int NT>
gnn_status launch_fast_for_k(const float *d_x, int64_t rows, int k, const float *d_w, int n, const XwEpilogue &ep,
                             float *d_z, hipStream_t s)
{
    if (k <= 32) return launch_fast<NT, 1>(d_x, rows, k, d_w, n, ep, d_z, s);
    if (k <= 64) return launch_fast<NT, 2>(d_x, rows, k, d_w, n, ep, d_z, s);
    if (k <= 96) return launch_fast<NT, 3>(d_x, rows, k, d_w, n, ep, d_z, s);
    return launch_fast<NT, 4>(d_x, rows, k, d_w, n, ep, d_z, s);
}

// Column tiles per wavefront (32 columns each: 1, 2 or 4).  Wide tiles read X once for all columns; narrow ones
// cut the work into more pieces, which matters when there are only a few tiles per SIMD: the cost of a choice is
// the largest number of 32-column tile products one SIMD gets, ties going to the wider tile.
int choose_column_tiles(int64_t rows, int n)
{
    const int64_t tiles = gnn_div_up(rows, kRowsPerWave);
    const int64_t simds = 4 * (int64_t)device_cu_count();
    const int widest = n <= 32 ? 1 : (n <= 64 ? 2 : 4);
    int best = widest;
    int64_t best_cost = 0;
    for (int nt = widest; nt >= 1; nt >>= 1) {
        const int64_t units = tiles * gnn_div_up(n, 32 * nt);
        const int64_t cost = gnn_div_up(units, simds) * nt;
        if (nt == widest || cost < best_cost) {
            best = nt;
            best_cost = cost;
        }
    }
    return best;
}

}  // namespace

static bool takes_fast_kernel(const float *d_x, int32_t k, const float *d_w, int32_t n)
{
    const bool x_vec4 = (k % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_x) & 15u) == 0);
    const bool w_vec4 = (n % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_w) & 15u) == 0);
    return x_vec4 && w_vec4 && k <= 2 * kSlab;   // w_vec4 implies n % 4 == 0
}

bool gnn_xw_takes_column_norm(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n)
{
    return rows > 0 && k > 0 && n > 0 && takes_fast_kernel(d_x, k, d_w, n);
}

bool gnn_xw_takes_transposed_w(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n)
{
    return rows > 0 && k > 0 && n > 0 && takes_fast_kernel(d_x, k, d_w, n);
}

gnn_status gnn_launch_xw(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                         const float *d_row_scale, const float *d_bias, bool relu, float *d_z, hipStream_t s,
                         const gnn_column_norm *norm, bool w_transposed)
{
    if (!d_x || !d_w || !d_z) return GNN_ERR_NULL;
    if (rows < 0 || k <= 0 || n <= 0) return GNN_ERR_BAD_SIZE;
    if (rows == 0) return GNN_OK;
    XwEpilogue ep;
    ep.row_scale = d_row_scale;
    ep.bias = d_bias;
    ep.relu = relu ? 1 : 0;
    if (norm) {
        if (!norm->mean || !norm->var || !d_row_scale || !takes_fast_kernel(d_x, k, d_w, n)) return GNN_ERR_UNSUPPORTED;
        ep.norm = *norm;
    }
    if (w_transposed) {
        if (!takes_fast_kernel(d_x, k, d_w, n)) return GNN_ERR_UNSUPPORTED;
        ep.w_transposed = 1;
    }
    const bool x_vec4 = (k % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_x) & 15u) == 0);
    const bool w_vec4 = (n % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_w) & 15u) == 0);
    if (takes_fast_kernel(d_x, k, d_w, n)) {
        switch (choose_column_tiles(rows, n)) {
        case 1: return launch_fast_for_k<1>(d_x, rows, k, d_w, n, ep, d_z, s);
        case 2: return launch_fast_for_k<2>(d_x, rows, k, d_w, n, ep, d_z, s);
        default: return launch_fast_for_k<4>(d_x, rows, k, d_w, n, ep, d_z, s);
        }
    }
    // General kernel.  Column tile: 64 or 32 if it divides n, else 128 wide when n is large enough, else the
    // smallest multiple of 32 covering n.
    int nt = n > 96 ? 4 : (n + 31) / 32;
    if (n % 64 == 0) nt = 2;
    else if (n % 32 == 0) nt = 1;
    switch (nt) {
    case 1: return launch_general<1>(d_x, rows, k, d_w, n, ep, d_z, x_vec4, w_vec4, 0, s);
    case 2: return launch_general<2>(d_x, rows, k, d_w, n, ep, d_z, x_vec4, w_vec4, 0, s);
    case 3: return launch_general<3>(d_x, rows, k, d_w, n, ep, d_z, x_vec4, w_vec4, 0, s);
    default: return launch_general<4>(d_x, rows, k, d_w, n, ep, d_z, x_vec4, w_vec4, 0, s);
    }
}

extern "C" gnn_status gnn_dense_xw(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                                   const float *d_row_scale, float *d_z, void *stream)
{
    return gnn_launch_xw(d_x, rows, k, d_w, n, d_row_scale, nullptr, false, d_z, static_cast<hipStream_t>(stream));
}
