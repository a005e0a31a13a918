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
constexpr int kFastWaves = 12, kFastThreads = 64 * kFastWaves;   // fast kernel: one block fills a compute unit
constexpr int kRowsPerWave = 32;
constexpr int kRowsPerBlock = 4 * kRowsPerWave;
constexpr int kSlab = 64;             // k-values per X register buffer / per staged W slab in the fallback

// What the store does after the product: optional per-row scale, per-column bias, relu (in that order).
struct XwEpilogue {
    const float *row_scale = nullptr;
    const float *bias = nullptr;
    int relu = 0;
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
__device__ __forceinline__ int w_lds_index(int col, int k, int kp)
{
    return col * kp + ((((k >> 2) ^ (col & 7)) << 2) | (k & 3));
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

    __device__ __forceinline__ void load(const float *__restrict__ w, int k, int n, int k0, int n0)
    {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int idx = min((int)threadIdx.x + it * NTHREADS, TOTAL - 1);   // a last, partial pass loads something valid
            int kk, c;
            decode(idx, kk, c);
            const bool inside = k0 + kk < k && n0 + c < n;
            const float *p = inside ? w + (int64_t)(k0 + kk) * n + n0 + c : w;
            v[it] = *reinterpret_cast<const float4 *>(p);
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

// Fast path: k <= 64*NSUB <= 128, k and n multiples of 4, 16-byte aligned rows (a ragged last row tile
// is handled by clamped loads and a guarded store, a ragged last column block by zero-filled W and a
// guarded store).  One block of twelve wavefronts per compute unit (three per SIMD, what the registers allow):
// it stages its columns of W once -- one copy in LDS serves all twelve -- and then every wavefront walks over
// 32-row tiles on its own.  Per tile a wavefront issues all of its X loads (no branches), runs the MFMAs and
// writes the tile with 128-bit stores; the wavefronts of a SIMD overlap one another's load latency with MFMAs
// (register use is kept low for that: no second X buffer).
// One wave tile of the fast kernel: 32 rows x NCB column blocks from the X fragments in registers.  They stay
// there while the column blocks are worked off one after the other (one accumulator set, reused): X is read
// once for NCB * BN output columns.
template <int NT, int NSUB, int NCB, int KSTEPS>
__device__ __forceinline__ void fast_wave_tile(const AFrag (&a)[NSUB], const float *ws, float sc, int64_t row,
                                               int64_t rows, int n, int n0, int r, int half,
                                               const float *__restrict__ bias, int relu, float *__restrict__ z)
{
    constexpr int BN = NT * 32;
    constexpr int KP = NSUB * kSlab;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
        floatx16 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub)
            mfma_subslab<NT, KSTEPS>(acc, a[sub], ws + cb * BN * KP, KP, sub * kSlab + 4 * KSTEPS * half, r);

        if (row < rows) {   // false only for lanes past the end in a ragged last tile
            float *zrow = z + row * n + n0 + cb * BN + 4 * half;
            const int ncols = n - n0 - cb * BN - 4 * half;   // n % 4 == 0: a group of four columns is inside or outside as a whole
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    if (t * 32 + 8 * g < ncols) {
                        float4 o = make_float4(acc[t][4 * g] * sc, acc[t][4 * g + 1] * sc, acc[t][4 * g + 2] * sc,
                                               acc[t][4 * g + 3] * sc);
                        if (bias) {   // n % 4 == 0 and the group lies inside: four bias values are there
                            const float *bp = bias + n0 + cb * BN + 4 * half + t * 32 + 8 * g;
                            o.x += bp[0]; o.y += bp[1]; o.z += bp[2]; o.w += bp[3];
                        }
                        if (relu) o = make_float4(fmaxf(o.x, 0.0f), fmaxf(o.y, 0.0f), fmaxf(o.z, 0.0f), fmaxf(o.w, 0.0f));
                        *reinterpret_cast<float4 *>(zrow + t * 32 + 8 * g) = o;
                    }
        }
    }
}

template <int NT, int NSUB, int NCB, bool SCALED, int KSTEPS>
__global__ __launch_bounds__(kFastThreads) void xw_fast_kernel(const float *__restrict__ x, int k,
                                                               const float *__restrict__ w, int n,
                                                               const float *__restrict__ row_scale,
                                                               const float *__restrict__ bias, int relu,
                                                               float *__restrict__ z, int64_t rows)
{
    constexpr int BN = NT * 32;
    constexpr int KP = NSUB * kSlab;
    // W is staged by the first kStageThreads threads: the number of 16-byte groups (a power of two) is a
    // multiple of it, so every staging thread makes the same number of passes and all loads go out at once.
    constexpr int kStageThreads = (KP * BN * NCB / 4) < 512 ? (KP * BN * NCB / 4) : 512;
    static_assert((KP * BN * NCB / 4) % kStageThreads == 0 && kStageThreads <= kFastThreads, "staging passes");
    extern __shared__ __align__(16) float ws[];   // [NCB * BN][KP], swizzled
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, half = lane >> 5;
    const int n0 = blockIdx.y * (BN * NCB);
    const int64_t num_wave_tiles = (rows + kRowsPerWave - 1) / kRowsPerWave;

    // Wave tile numbers go round the blocks first, then round the wavefronts of a block, so that a last, partly
    // filled round puts one tile on as many compute units as possible.
    const int64_t wt_stride = (int64_t)gridDim.x * kFastWaves;
    int64_t wt = (int64_t)wave * gridDim.x + blockIdx.x;
    int64_t row = wt * kRowsPerWave + r;

    // W's loads are issued first, then the first tile's X loads (clamped addresses: safe also for a wavefront
    // without a tile), which stay in flight while W is written to LDS: loads return in order, so waiting for W
    // does not wait for X.
    AFrag a[NSUB];
    float sc = 1.0f;
    {
        WStage<BN * NCB, KP, kStageThreads> st;
        const bool stager = threadIdx.x < kStageThreads;   // whole wavefronts
        if (stager) st.load(w, k, n, 0, n0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) load_a<true, KSTEPS>(a[sub], x, rows, k, row, sub * kSlab, half);
        if constexpr (SCALED) sc = row_scale[min(row, rows - 1)];
        __builtin_amdgcn_sched_barrier(0);
        if (stager) st.store(ws, k, n, 0, n0);
    }
    __syncthreads();

    // From here on the wavefronts are independent.  The first tile (already loaded) is peeled off the loop.
    if (wt < num_wave_tiles) fast_wave_tile<NT, NSUB, NCB, KSTEPS>(a, ws, sc, row, rows, n, n0, r, half, bias, relu, z);
    for (wt += wt_stride; wt < num_wave_tiles; wt += wt_stride) {
        row = wt * kRowsPerWave + r;
#pragma unroll
        for (int sub = 0; sub < NSUB; ++sub) load_a<true, KSTEPS>(a[sub], x, rows, k, row, sub * kSlab, half);
        if constexpr (SCALED) sc = row_scale[min(row, rows - 1)];
        fast_wave_tile<NT, NSUB, NCB, KSTEPS>(a, ws, sc, row, rows, n, n0, r, half, bias, relu, z);
    }
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

template <int NT, int NSUB, int NCB, int KSTEPS = 8>
gnn_status launch_fast(const float *d_x, int64_t rows, int k, const float *d_w, int n, const XwEpilogue &ep,
                       float *d_z, hipStream_t s)
{
    constexpr int BN = NT * 32 * NCB;   // output columns per block
    const int64_t wave_tiles = gnn_div_up(rows, kRowsPerWave);
    const size_t lds = (size_t)NSUB * kSlab * BN * sizeof(float);
    // One resident block per compute unit (fewer where there are several column blocks or few rows: then at
    // least one wave tile per block, so that small inputs still spread over the chip).
    const int col_blocks = (int)gnn_div_up(n, BN);
    const int64_t blocks = std::max<int64_t>(1, std::min<int64_t>(device_cu_count() / col_blocks, wave_tiles));
    const dim3 grid((unsigned)blocks, (unsigned)col_blocks);
    if (ep.row_scale)
        hipLaunchKernelGGL((xw_fast_kernel<NT, NSUB, NCB, true, KSTEPS>), grid, dim3(kFastThreads), lds, s, d_x, k, d_w, n,
                           ep.row_scale, ep.bias, ep.relu, d_z, rows);
    else
        hipLaunchKernelGGL((xw_fast_kernel<NT, NSUB, NCB, false, KSTEPS>), grid, dim3(kFastThreads), lds, s, d_x, k, d_w, n,
                           ep.row_scale, ep.bias, ep.relu, d_z, rows);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

template <int NT, int NCB>
gnn_status launch_fast_for_k(const float *d_x, int64_t rows, int k, const float *d_w, int n, const XwEpilogue &ep,
                             float *d_z, hipStream_t s)
{
    // up to 64 k-values: one sub-slab of 16, 32 or 64 (two, four or eight steps); up to 128: two full sub-slabs
    if (k <= 16) return launch_fast<NT, 1, NCB, 2>(d_x, rows, k, d_w, n, ep, d_z, s);
    if (k <= 32) return launch_fast<NT, 1, NCB, 4>(d_x, rows, k, d_w, n, ep, d_z, s);
    if (k <= kSlab) return launch_fast<NT, 1, NCB, 8>(d_x, rows, k, d_w, n, ep, d_z, s);
    return launch_fast<NT, 2, NCB, 8>(d_x, rows, k, d_w, n, ep, d_z, s);
}

}  // namespace

gnn_status gnn_launch_xw(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                         const float *d_row_scale, const float *d_bias, bool relu, float *d_z, hipStream_t s)
{
    if (!d_x || !d_w || !d_z) return GNN_ERR_NULL;
    if (rows < 0 || k <= 0 || n <= 0) return GNN_ERR_BAD_SIZE;
    if (rows == 0) return GNN_OK;
    XwEpilogue ep;
    ep.row_scale = d_row_scale;
    ep.bias = d_bias;
    ep.relu = relu ? 1 : 0;
    const bool x_vec4 = (k % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_x) & 15u) == 0);
    const bool w_vec4 = (n % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_w) & 15u) == 0);
    if (x_vec4 && w_vec4 && k <= 2 * kSlab) {   // w_vec4 implies n % 4 == 0
        // column tiles of 32 (n <= 32) or 64, two of them per block where the matrix is wider than one
        if (n <= 32) return launch_fast_for_k<1, 1>(d_x, rows, k, d_w, n, ep, d_z, s);
        if (n <= 64) return launch_fast_for_k<2, 1>(d_x, rows, k, d_w, n, ep, d_z, s);
        return launch_fast_for_k<2, 2>(d_x, rows, k, d_w, n, ep, d_z, s);
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
