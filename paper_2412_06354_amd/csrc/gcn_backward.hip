// Backward of GCNConv (the layer of the paper's training example, which is differentiated end to
// end).  With Ahat = D^-1/2 (A [+ I]) D^-1/2 and G = dL/d out:
//     T = Ahat^T G,    dL/dX = T W^T,    dL/dW = X^T T,    dL/db = column sums of G.
//   * T is a propagate over the graph sorted by source: rows of G are gathered with the destination
//     side factor as a weight looked up per edge (G is never rescaled in memory), summed, and the epilogue
//     adds the self-loop term and applies the source side factor -- the forward's fused kernel run on the
//     transposed topology (the degree factors always come from the forward graph's in-degrees);
//   * T W^T is the MFMA projection kernel, which stages W transposed anyway and reads the forward's W as it is
//     (shapes that kernel does not take go through a transposed copy of W);
//   * X^T T contracts over the N rows: v_mfma_f32_32x32x2_f32 consumes two rows per instruction and
//     both operands are read along rows (coalesced); row chunks give partial [f_in x f_out] blocks
//     that a second kernel adds up in chunk order (deterministic);
//   * the bias gradient uses the same two-stage scheme.
// A layer that widens (f_in < f_out) is differentiated in the order its forward runs in, so that both gathers move
// rows of f_in values:   dL/dW = (Ahat X)^T G  (Ahat X recomputed by the forward's narrow propagate),
// dL/dX = Ahat^T (G W^T)  (projection first, destination-side factor in its store, then the propagate by source).
#include "gnn_internal.h"

#include <algorithm>

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
constexpr int kThreads = 256;

// First stage of the bias gradient: partial[chunk][j] = sum over the chunk's rows of G[r][j].  A block owns a row
// chunk; its threads form (row slice, column group) pairs, a slice takes every `slices`-th row, and the slices'
// sums are folded through LDS in slice order.
template <int VEC>
__global__ __launch_bounds__(kThreads) void column_sums_partial_kernel(int64_t N, int F, const float *__restrict__ g,
                                                                       int64_t rows_per_chunk,
                                                                       float *__restrict__ partial)
{
    __shared__ float fold[kThreads * VEC];
    const int fv = F / VEC;
    const int width = min(fv, kThreads), slices = kThreads / width;
    const int cg0 = threadIdx.x % width, sl = threadIdx.x / width;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk, r1 = min(N, r0 + rows_per_chunk);
    for (int cbase = 0; cbase < fv; cbase += width) {
        const int cg = cbase + cg0;
        const bool active = sl < slices && cg < fv;
        float sum[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) sum[c] = 0.0f;
        if (active) {
#pragma unroll 4
            for (int64_t r = r0 + sl; r < r1; r += slices) {
                float v[VEC];
                if constexpr (VEC == 4) {
                    const float4 t = *reinterpret_cast<const float4 *>(g + r * F + cg * 4);
                    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
                } else {
                    v[0] = g[r * F + cg];
                }
#pragma unroll
                for (int c = 0; c < VEC; ++c) sum[c] += v[c];
            }
        }
        {
#pragma unroll
            for (int c = 0; c < VEC; ++c) fold[threadIdx.x * VEC + c] = sum[c];
            __syncthreads();
            if (sl == 0 && cg < fv) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    float t = 0.0f;
                    for (int q = 0; q < slices; ++q) t += fold[(q * width + cg0) * VEC + c];
                    partial[(int64_t)blockIdx.x * F + cg * VEC + c] = t;
                }
            }
            __syncthreads();
        }
    }
}

__global__ __launch_bounds__(kThreads) void transpose_kernel(const float *__restrict__ w, int rows, int cols,
                                                             float *__restrict__ wt)
{
    const int idx = blockIdx.x * kThreads + threadIdx.x;
    if (idx >= rows * cols) return;
    const int r = idx / cols, c = idx - r * cols;
    wt[c * rows + r] = w[idx];
}

// partial[chunk][i][j] = sum over the chunk's rows of X[row][i] * Y[row][j].
// A block of 4 wavefronts covers STRIPS (1, 2 or 4) 32-wide strips of i and all its columns j in NT accumulator
// tiles of 32; with fewer than four strips the spare wavefronts take every other (every fourth) batch of rows
// of the chunk and their tiles are added through LDS in a fixed order at the end.  The kernel lives on loads in
// flight -- one MFMA consumes two rows of both operands in 64 cycles, a memory round trip takes thousands --
// hence two register sets of U row pairs each and all four wavefronts at work.
template <int NT, int STRIPS>
__global__ __launch_bounds__(kThreads) void xty_partial_kernel(const float *__restrict__ x, const float *__restrict__ y,
                                                               int64_t rows, int f_in, int f_out,
                                                               int64_t rows_per_chunk, float *__restrict__ partial)
{
    constexpr int U = NT >= 4 ? 4 : 8;   // row pairs per register set
    constexpr int RG = 4 / STRIPS;       // row groups
    __shared__ float red[RG > 1 ? (RG - 1) * STRIPS * NT * 1024 : 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, kk = lane >> 5;
    const int strip = wave % STRIPS, rg = wave / STRIPS;
    const int i0 = (blockIdx.y * STRIPS + strip) * 32;
    const int j0 = blockIdx.z * NT * 32;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk, r1 = min(rows, r0 + rows_per_chunk);
    const bool active = i0 < f_in && r0 < r1;   // wavefront-uniform

    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    if (active) {
        // Batch s covers the rows r0 + 2 U s ... ; row group rg takes the batches s = rg, rg + RG, ...
        auto load_set = [&](float (&a)[U], float (&b)[U][NT], int64_t s) {
            const int64_t rp = r0 + s * (2 * U);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // Unconditional loads from clamped addresses, no branches between them.  A row past the chunk is
                // cancelled by a zero factor on the X side alone (inputs are finite by contract); columns past
                // the matrices only feed accumulator entries that are never stored.
                const int64_t row = rp + 2 * u + kk;
                const int64_t rc = min(row, r1 - 1);
                a[u] = x[rc * f_in + min(i0 + c, f_in - 1)] * (row < r1 ? 1.0f : 0.0f);
#pragma unroll
                for (int t = 0; t < NT; ++t) b[u][t] = y[rc * f_out + min(j0 + t * 32 + c, f_out - 1)];
            }
        };
        auto mfma_set = [&](const float (&a)[U], const float (&b)[U][NT]) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u][t], acc[t], 0, 0, 0);
        };
        float a0[U], b0[U][NT], a1[U], b1[U][NT];
        load_set(a0, b0, rg);
        for (int64_t s = rg; r0 + s * (2 * U) < r1; s += 2 * RG) {
            load_set(a1, b1, s + RG);
            mfma_set(a0, b0);
            load_set(a0, b0, s + 2 * RG);
            mfma_set(a1, b1);
        }
    }
    if constexpr (RG > 1) {   // the spare row groups hand their tiles to group 0, which adds them in group order
        if (active && rg > 0) {
            float *mine = red + ((rg - 1) * STRIPS + strip) * NT * 1024;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) mine[(t * 16 + v) * 64 + lane] = acc[t][v];
        }
        __syncthreads();
        if (active && rg == 0) {
#pragma unroll
            for (int q = 1; q < RG; ++q) {
                const float *theirs = red + ((q - 1) * STRIPS + strip) * NT * 1024;
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[t][v] += theirs[(t * 16 + v) * 64 + lane];
            }
        }
    }
    if (i0 < f_in && rg == 0) {   // an empty trailing chunk still writes its zeros: the sum over chunks reads them
        // accumulator register v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32
        float *out = partial + (int64_t)blockIdx.x * f_in * f_out;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = i0 + 8 * (v / 4) + 4 * kk + (v % 4);
                const int j = j0 + t * 32 + c;
                if (i < f_in && j < f_out) out[(int64_t)i * f_out + j] = acc[t][v];
            }
    }
}

// The same contraction with both operands staged through LDS, for shapes whose rows are read as 128-bit pieces
// (f_in, f_out multiples of 4, aligned arrays).  A block of four wavefronts (2 x 2) owns a row chunk and an output
// tile of 2*TI*32 x 2*TJ*32; it walks the chunk in steps of kXtyRows rows: every thread loads its 16-byte pieces of
// the next step's rows of X and Y (whole rows of the tile: coalesced, and each line is requested once per block
// instead of once per wavefront), the pieces of the current step are written to LDS, and each wavefront reads its
// MFMA operands from there -- lane (c, kk) takes column c of row 2m + kk, a conflict-free 32-bit read because the
// LDS rows are padded by 32 floats.  The loads of a step have the whole MFMA work of the previous step to arrive
// (a second register set, loads two steps ahead, changed nothing).
constexpr int kXtyRows = 32;   // rows per step
constexpr int kXtyPad = 32;    // floats between LDS rows: the two row halves of a read fall on different banks

template <int COLS>   // columns of the staged tile
struct XtyStage {
    static constexpr int kPiecesPerRow = COLS / 4;
    static constexpr int kRowsPerPass = kThreads / kPiecesPerRow;
    static constexpr int kPasses = kXtyRows / kRowsPerPass;
    static_assert(kThreads % kPiecesPerRow == 0 && kXtyRows % kRowsPerPass == 0, "stage shape");
    float4 v[kPasses];

    // rows [r, r + kXtyRows) of the chunk ending at r1, columns [c0, c0 + COLS) of a matrix with f columns
    __device__ __forceinline__ void load(const float *__restrict__ m, int64_t r, int64_t r1, int f, int c0)
    {
        const int piece = threadIdx.x % kPiecesPerRow, row = threadIdx.x / kPiecesPerRow;
        const int col = c0 + piece * 4;
#pragma unroll
        for (int q = 0; q < kPasses; ++q) {
            const int64_t rr = r + q * kRowsPerPass + row;
            v[q] = make_float4(0.f, 0.f, 0.f, 0.f);   // rows past the chunk and columns past the matrix add nothing
            if (rr < r1 && col < f) v[q] = *reinterpret_cast<const float4 *>(m + rr * f + col);
        }
    }
    __device__ __forceinline__ void store(float *lds) const
    {
        const int piece = threadIdx.x % kPiecesPerRow, row = threadIdx.x / kPiecesPerRow;
#pragma unroll
        for (int q = 0; q < kPasses; ++q)
            *reinterpret_cast<float4 *>(lds + (q * kRowsPerPass + row) * (COLS + kXtyPad) + piece * 4) = v[q];
    }
};

template <int TI, int TJ>
__global__ __launch_bounds__(kThreads) void xty_staged_kernel(const float *__restrict__ x, const float *__restrict__ y,
                                                              int64_t rows, int f_in, int f_out,
                                                              int64_t rows_per_chunk, float *__restrict__ partial)
{
    constexpr int BI = 2 * TI * 32, BJ = 2 * TJ * 32;
    __shared__ __align__(16) float xs[kXtyRows * (BI + kXtyPad)];
    __shared__ __align__(16) float ys[kXtyRows * (BJ + kXtyPad)];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 31, kk = lane >> 5;
    const int wi = wave & 1, wj = wave >> 1;
    const int i0 = blockIdx.y * BI, j0 = blockIdx.z * BJ;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk, r1 = min(rows, r0 + rows_per_chunk);

    floatx16 acc[TI][TJ];
#pragma unroll
    for (int a = 0; a < TI; ++a)
#pragma unroll
        for (int b = 0; b < TJ; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    const float *xa = xs + kk * (BI + kXtyPad) + wi * TI * 32 + c;
    const float *yb = ys + kk * (BJ + kXtyPad) + wj * TJ * 32 + c;
    auto row_pair = [&](int m) {
        float a[TI], b[TJ];
#pragma unroll
        for (int ti = 0; ti < TI; ++ti) a[ti] = xa[2 * m * (BI + kXtyPad) + ti * 32];
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj) b[tj] = yb[2 * m * (BJ + kXtyPad) + tj * 32];
#pragma unroll
        for (int ti = 0; ti < TI; ++ti)
#pragma unroll
            for (int tj = 0; tj < TJ; ++tj)
                acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ti], b[tj], acc[ti][tj], 0, 0, 0);
    };
    XtyStage<BI> sx;
    XtyStage<BJ> sy;
    if (r0 < r1) {
        sx.load(x, r0, r1, f_in, i0);
        sy.load(y, r0, r1, f_out, j0);
    }
    for (int64_t r = r0; r < r1; r += kXtyRows) {   // the same trip count for every thread of the block
        __syncthreads();                           // the previous step's operand reads are done
        sx.store(xs);
        sy.store(ys);
        __syncthreads();
        if (r + kXtyRows < r1) {                    // in flight during this step's MFMAs
            sx.load(x, r + kXtyRows, r1, f_in, i0);
            sy.load(y, r + kXtyRows, r1, f_out, j0);
        }
        if (r + kXtyRows <= r1) {
#pragma unroll 2
            for (int m = 0; m < kXtyRows / 2; ++m) row_pair(m);
        } else {   // a short last step does no work on its zero rows
            const int pairs = ((int)(r1 - r) + 1) / 2;
            for (int m = 0; m < pairs; ++m) row_pair(m);
        }
    }
    // accumulator register v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32; an empty trailing chunk
    // still writes its zeros (the sum over chunks reads them)
    float *out = partial + (int64_t)blockIdx.x * f_in * f_out;
#pragma unroll
    for (int ti = 0; ti < TI; ++ti)
#pragma unroll
        for (int tj = 0; tj < TJ; ++tj)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = i0 + (wi * TI + ti) * 32 + 8 * (v / 4) + 4 * kk + (v % 4);
                const int j = j0 + (wj * TJ + tj) * 32 + c;
                if (i < f_in && j < f_out) out[(int64_t)i * f_out + j] = acc[ti][tj][v];
            }
}

// out[q] = factor * sum over chunks of partial[chunk][q], in a fixed order: a block owns 64 elements, its SLICES
// thread rows take the chunks round-robin (eight loads in flight each) and are folded through LDS in slice order.
// SLICES = 16 where there are few elements (few blocks) and many chunks: the chain of dependent adds is what
// takes the time there.
template <int SLICES>
__global__ __launch_bounds__(64 * SLICES) void sum_partials_kernel(const float *__restrict__ partial, int chunks,
                                                                   int64_t elems, float factor, float *__restrict__ out)
{
    __shared__ float fold[SLICES][64];
    const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
    const int64_t q = (int64_t)blockIdx.x * 64 + lane;
    float s = 0.0f;
    if (q < elems) {
        int ch = slice;
        for (; ch + 7 * SLICES < chunks; ch += 8 * SLICES) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(ch + SLICES * u) * elems + q];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; ch < chunks; ch += SLICES) s += partial[(int64_t)ch * elems + q];
    }
    fold[slice][lane] = s;
    __syncthreads();
    if (slice == 0 && q < elems) {
        float t = 0.0f;
        if constexpr (SLICES == 4) {
            t = (fold[0][lane] + fold[1][lane]) + (fold[2][lane] + fold[3][lane]);
        } else {
#pragma unroll
            for (int k = 0; k < SLICES; ++k) t += fold[k][lane];
        }
        out[q] = factor == 1.0f ? t : t * factor;
    }
}

// The same sum for few elements and many chunks: a block of 1024 threads owns eight elements, its 128 thread
// rows take the chunks round-robin (eight loads in flight each) and are added through LDS by a fixed halving
// tree -- the chain of dependent adds, which is what takes the time here, is chunks / 128 + 7 long.
constexpr int kTreeThreads = 1024, kTreeCols = 8, kTreeSlots = kTreeThreads / kTreeCols;

__global__ __launch_bounds__(kTreeThreads) void sum_partials_tree_kernel(const float *__restrict__ partial, int chunks,
                                                                         int64_t elems, float factor,
                                                                         float *__restrict__ out)
{
    __shared__ float fold[kTreeSlots][kTreeCols];
    const int c0 = threadIdx.x % kTreeCols, slot = threadIdx.x / kTreeCols;
    const int64_t q = (int64_t)blockIdx.x * kTreeCols + c0;
    const bool ok = q < elems;
    const int64_t qc = ok ? q : 0;
    float s = 0.0f;
    int ch = slot;
    for (; ch + 7 * kTreeSlots < chunks; ch += 8 * kTreeSlots) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(ch + kTreeSlots * u) * elems + qc];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; ch < chunks; ch += kTreeSlots) s += partial[(int64_t)ch * elems + qc];
    fold[slot][c0] = s;
    __syncthreads();
#pragma unroll
    for (int h = kTreeSlots / 2; h >= 1; h >>= 1) {
        if (slot < h) fold[slot][c0] += fold[slot + h][c0];
        __syncthreads();
    }
    if (slot == 0 && ok) {
        const float t = fold[0][c0];
        out[q] = factor == 1.0f ? t : t * factor;
    }
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

int chunk_count(int64_t rows) { return gnn_row_chunk_count(rows); }

struct BackwardLayout {
    size_t gs, t, wt, part, total;
};

BackwardLayout layout(int64_t N, int f_in, int f_out)
{
    BackwardLayout l{};
    const size_t nf = align256((size_t)N * f_out * sizeof(float));
    const int chunks = chunk_count(N);
    l.gs = 0;
    l.t = nf;
    l.wt = 2 * nf;
    l.part = l.wt + align256((size_t)f_in * f_out * sizeof(float));
    l.total = l.part + align256((size_t)chunks * std::max(f_in, 1) * f_out * sizeof(float));
    return l;
}

}  // namespace

int gnn_row_chunk_count(int64_t rows)
{
    // About 256 rows per chunk, at most 2048 chunks.  Above one chunk per compute unit the count is rounded up
    // to a multiple of 256, so that blocks working on one chunk each come in whole rounds over the chip; below,
    // chunks shrink to as few as 32 rows so that small inputs still spread over many blocks (a block's walk over
    // its rows is a chain of dependent memory round trips).
    int64_t c = std::max<int64_t>(1, gnn_div_up(rows, 256));
    if (c > 256) c = gnn_div_up(c, 256) * 256;
    else c = std::min<int64_t>(256, std::max<int64_t>(1, gnn_div_up(rows, 32)));
    return (int)std::min<int64_t>(2048, c);
}

gnn_status gnn_launch_sum_partials_scaled(const float *d_partial, int chunks, int64_t elems, float factor,
                                          float *d_out, hipStream_t s)
{
    if (elems <= 0) return GNN_OK;
    const dim3 grid((unsigned)gnn_div_up(elems, 64));
    if (elems <= 4096 && chunks >= 64)
        hipLaunchKernelGGL(sum_partials_tree_kernel, dim3((unsigned)gnn_div_up(elems, kTreeCols)), dim3(kTreeThreads), 0,
                           s, d_partial, chunks, elems, factor, d_out);
    else
        hipLaunchKernelGGL(sum_partials_kernel<4>, grid, dim3(64 * 4), 0, s, d_partial, chunks, elems, factor, d_out);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_launch_sum_partials(const float *d_partial, int chunks, int64_t elems, float *d_out, hipStream_t s)
{
    return gnn_launch_sum_partials_scaled(d_partial, chunks, elems, 1.0f, d_out, s);
}

template <int NT, int STRIPS>
static gnn_status launch_xty_shape(const float *d_x, const float *d_y, int64_t rows, int f_in, int f_out, int chunks,
                                   float *d_partial, hipStream_t s)
{
    const int64_t rows_per_chunk = gnn_div_up(rows, chunks);
    const dim3 grid((unsigned)chunks, (unsigned)gnn_div_up(f_in, 32 * STRIPS), (unsigned)gnn_div_up(f_out, NT * 32));
    hipLaunchKernelGGL((xty_partial_kernel<NT, STRIPS>), grid, dim3(kThreads), 0, s, d_x, d_y, rows, f_in, f_out,
                       rows_per_chunk, d_partial);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

template <int NT>
static gnn_status launch_xty_tiles(const float *d_x, const float *d_y, int64_t rows, int f_in, int f_out, int chunks,
                                   float *d_partial, hipStream_t s)
{
    if (f_in <= 32) return launch_xty_shape<NT, 1>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s);
    if (f_in <= 64) return launch_xty_shape<NT, 2>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s);
    return launch_xty_shape<NT, 4>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s);
}

template <int TI, int TJ>
static gnn_status launch_xty_staged(const float *d_x, const float *d_y, int64_t rows, int f_in, int f_out, int chunks,
                                    float *d_partial, hipStream_t s)
{
    const int64_t rows_per_chunk = gnn_div_up(rows, chunks);
    const dim3 grid((unsigned)chunks, (unsigned)gnn_div_up(f_in, 2 * TI * 32), (unsigned)gnn_div_up(f_out, 2 * TJ * 32));
    hipLaunchKernelGGL((xty_staged_kernel<TI, TJ>), grid, dim3(kThreads), 0, s, d_x, d_y, rows, f_in, f_out,
                       rows_per_chunk, d_partial);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_launch_xty(const float *d_x, const float *d_y, int64_t rows, int f_in, int f_out, float *d_partial,
                          float *d_out, hipStream_t s)
{
    const int chunks = gnn_row_chunk_count(rows);
    // rows that can be read as 128-bit pieces and an output of at least 64 x 64: operands staged through LDS
    const bool pieces = f_in % 4 == 0 && f_out % 4 == 0 &&
                        ((reinterpret_cast<uintptr_t>(d_x) | reinterpret_cast<uintptr_t>(d_y)) & 15u) == 0;
    if (pieces && f_in > 32 && f_out > 32) {
        if (f_in > 64 && f_out > 64) GNN_TRY((launch_xty_staged<2, 2>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s)));
        else if (f_in > 64) GNN_TRY((launch_xty_staged<2, 1>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s)));
        else if (f_out > 64) GNN_TRY((launch_xty_staged<1, 2>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s)));
        else GNN_TRY((launch_xty_staged<1, 1>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s)));
        return gnn_launch_sum_partials(d_partial, chunks, (int64_t)f_in * f_out, d_out, s);
    }
    // a wavefront holds 1, 2 or 4 accumulator tiles of 32 columns: no MFMA work on columns that do not exist
    if (f_out <= 32) GNN_TRY(launch_xty_tiles<1>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s));
    else if (f_out <= 64) GNN_TRY(launch_xty_tiles<2>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s));
    else GNN_TRY(launch_xty_tiles<2>(d_x, d_y, rows, f_in, f_out, chunks, d_partial, s));   // wider: 64-column blocks
    return gnn_launch_sum_partials(d_partial, chunks, (int64_t)f_in * f_out, d_out, s);
}

gnn_status gnn_launch_transpose(const float *d_w, int rows, int cols, float *d_wt, hipStream_t s)
{
    hipLaunchKernelGGL(transpose_kernel, dim3((unsigned)gnn_div_up((int64_t)rows * cols, kThreads)), dim3(kThreads), 0,
                       s, d_w, rows, cols, d_wt);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_launch_xwt(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                          const float *d_row_scale, float *d_wt, float *d_z, hipStream_t s)
{
    if (gnn_xw_takes_transposed_w(d_x, rows, k, d_w, n))
        return gnn_launch_xw(d_x, rows, k, d_w, n, d_row_scale, nullptr, false, d_z, s, nullptr, true);
    GNN_TRY(gnn_launch_transpose(d_w, n, k, d_wt, s));
    return gnn_launch_xw(d_x, rows, k, d_wt, n, d_row_scale, nullptr, false, d_z, s);
}

extern "C" {

size_t gnn_gcnconv_backward_workspace_bytes(int32_t num_nodes, int32_t f_in, int32_t f_out)
{
    if (num_nodes <= 0 || f_in <= 0 || f_out <= 0) return 0;
    return layout(num_nodes, f_in, f_out).total;
}

gnn_status gnn_gcnconv_backward(const gnn_graph *g, const gnn_graph *g_by_source, const float *d_x, int32_t f_in,
                                const float *d_w, int32_t f_out, int32_t add_self_loops, const float *d_grad_out,
                                float *d_grad_x, float *d_grad_w, float *d_grad_b, void *d_workspace,
                                size_t workspace_bytes, void *stream)
{
    if (!g || !g_by_source || !d_grad_out || !d_workspace) return GNN_ERR_NULL;
    if (f_in <= 0 || f_out <= 0) return GNN_ERR_BAD_SIZE;
    if (g->bipartite) return GNN_ERR_UNSUPPORTED;   // one node set only
    if (g_by_source->num_nodes != g->num_nodes || g_by_source->num_edges != g->num_edges) return GNN_ERR_BAD_SIZE;
    if ((d_grad_x && !d_w) || (d_grad_w && !d_x)) return GNN_ERR_NULL;
    const int64_t N = g->num_nodes;
    const BackwardLayout l = layout(N, f_in, f_out);
    if (workspace_bytes < l.total) return GNN_ERR_BAD_SIZE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255u) return GNN_ERR_BAD_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(d_workspace);
    float *gs = reinterpret_cast<float *>(ws + l.gs), *t = reinterpret_cast<float *>(ws + l.t),
          *wt = reinterpret_cast<float *>(ws + l.wt),
          *part = reinterpret_cast<float *>(ws + l.part);
    const int chunks = chunk_count(N);
    const float *dinv = add_self_loops ? g->dinv_loop : g->dinv_plain;   // the forward graph's degree factors

    const bool narrow_first = f_in < f_out;   // the order gnn_gcnconv runs this shape in
    const bool need_t = !narrow_first && (d_grad_x || d_grad_w);
    if (d_grad_b) {
        // column sums of G in two stages (64-row chunks: enough blocks to stream at full rate; the partial sums fit
        // the workspace's partial-result area)
        const int64_t bias_chunks = std::max<int64_t>(
            1, std::min<int64_t>(std::min<int64_t>(2048, gnn_div_up(N, 64)), (int64_t)chunks * f_in));
        const int64_t bias_rows = gnn_div_up(N, bias_chunks);
        const dim3 grid((unsigned)gnn_div_up(N, bias_rows));
        const bool vec4 = f_out % 4 == 0 && (reinterpret_cast<uintptr_t>(d_grad_out) & 15u) == 0;
        if (vec4)
            hipLaunchKernelGGL(column_sums_partial_kernel<4>, grid, dim3(kThreads), 0, s, N, f_out, d_grad_out, bias_rows, part);
        else
            hipLaunchKernelGGL(column_sums_partial_kernel<1>, grid, dim3(kThreads), 0, s, N, f_out, d_grad_out, bias_rows, part);
        GNN_LAUNCH_CHECK();
        GNN_TRY(gnn_launch_sum_partials(part, (int)grid.x, (int64_t)f_out, d_grad_b, s));
    }
    if (narrow_first) {
        if (d_grad_w) {   // t = Ahat X [N x f_in], then (Ahat X)^T G
            gnn_epilogue agg;
            agg.self_scale = add_self_loops ? 1.0f : 0.0f;
            agg.row_scale = dinv;
            agg.source_scale = dinv;
            GNN_TRY(gnn_launch_propagate(g, d_x, f_in, nullptr, 1, GNN_EDGE_ORDER_CSR, GNN_MSG_COPY_XJ, 0, agg, t, s));
            GNN_TRY(gnn_launch_xty(t, d_grad_out, N, f_in, f_out, part, d_grad_w, s));
        }
        if (d_grad_x) {   // gs = dinv * (G W^T) [N x f_in], then the propagate over the transposed topology
            GNN_TRY(gnn_launch_xwt(d_grad_out, N, f_out, d_w, f_in, dinv, wt, gs, s));
            gnn_epilogue epi;
            epi.self_scale = add_self_loops ? 1.0f : 0.0f;
            epi.row_scale = dinv;
            GNN_TRY(gnn_launch_propagate(g_by_source, gs, f_in, nullptr, 1, GNN_EDGE_ORDER_CSR, GNN_MSG_COPY_XJ, 0,
                                         epi, d_grad_x, s));
        }
        return GNN_OK;
    }
    if (need_t) {
        gnn_epilogue epi;
        epi.self_scale = add_self_loops ? 1.0f : 0.0f;
        epi.row_scale = dinv;
        epi.source_scale = dinv;   // the gathered row's factor rides on the edge: G is never rescaled in memory
        GNN_TRY(gnn_launch_propagate(g_by_source, d_grad_out, f_out, nullptr, 1, GNN_EDGE_ORDER_CSR, GNN_MSG_COPY_XJ, 0,
                                     epi, t, s));
    }
    if (d_grad_x) {
        GNN_TRY(gnn_launch_xwt(t, N, f_out, d_w, f_in, nullptr, wt, d_grad_x, s));
    }
    if (d_grad_w) GNN_TRY(gnn_launch_xty(d_x, t, N, f_in, f_out, part, d_grad_w, s));
    return GNN_OK;
}

}  // extern "C"
