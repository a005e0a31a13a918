// The dense-side layers of the paper's example model (section 3, "Training Example": two graph convolutions with
// a batch normalisation and a relu in between, a mean readout per graph and a dense head) and the chain itself
// as one call:
//   * batch normalisation across the node dimension, with batch statistics (one pass over the rows with running
//     (mean, squared-deviation) pairs that merge exactly -- no cancellation; few rows: two passes in one launch)
//     or stored ones, optional relu fused;
//   * a dense layer act(X W + b) on the MFMA projection kernel;
//   * the forward chain, which only sequences entry points of this library on the caller's stream.
// Column statistics use the two-stage scheme of the backward passes: per-chunk partial results,
// then a fixed-order merge over chunks (deterministic, no atomics).
#include "gnn_internal.h"

#include <algorithm>

namespace {

constexpr int kThreads = 256;

// One pass over x for both statistics.  Running (count, mean, sum of squared deviations) per thread in the
// single-pass form that does not cancel (each value updates the mean and adds (x - old mean)(x - new mean)); two
// such triples over disjoint row sets merge exactly:
//     n = na + nb,  delta = mb - ma,  m = ma + delta nb / n,  q = qa + qb + delta^2 na nb / n.
// Threads, then chunks, are merged in a fixed order: deterministic, and x is read once instead of twice.
struct Moments {
    float n, m, q;
};

__device__ __forceinline__ void moments_add(Moments &a, float v)
{
    a.n += 1.0f;
    const float d = v - a.m;
    a.m += d * __builtin_amdgcn_rcpf(a.n);
    a.q = fmaf(d, v - a.m, a.q);
}

__device__ __forceinline__ void moments_merge(Moments &a, const Moments &b)
{
    if (b.n == 0.0f) return;
    const float n = a.n + b.n, delta = b.m - a.m, w = b.n * __builtin_amdgcn_rcpf(n);   // weight to within an ulp
    a.m = fmaf(delta, w, a.m);
    a.q = a.q + b.q + delta * delta * (a.n * w);
    a.n = n;
}

// part_m[chunk][f], part_q[chunk][f]: mean and sum of squared deviations of the chunk's rows (the count follows from
// the chunk's bounds).
__global__ __launch_bounds__(kThreads) void column_moments_partial_kernel(const float *__restrict__ x, int64_t N, int F,
                                                                          int64_t rows_per_chunk,
                                                                          float *__restrict__ part_m,
                                                                          float *__restrict__ part_q)
{
    __shared__ float fn[kThreads], fm[kThreads], fq[kThreads];
    const int cw = min(F, kThreads), slices = kThreads / cw;
    const int rs = threadIdx.x / cw, c0 = threadIdx.x % cw;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk, r1 = min(N, r0 + rows_per_chunk);
    for (int cbase = 0; cbase < F; cbase += cw) {
        const int col = cbase + c0;
        Moments a{0.0f, 0.0f, 0.0f};
        if (rs < slices && col < F) {
#pragma unroll 4
            for (int64_t row = r0 + rs; row < r1; row += slices) moments_add(a, x[row * F + col]);
        }
        fn[threadIdx.x] = a.n;
        fm[threadIdx.x] = a.m;
        fq[threadIdx.x] = a.q;
        __syncthreads();
        if (rs == 0 && col < F) {
            for (int s = 1; s < slices; ++s) moments_merge(a, Moments{fn[s * cw + c0], fm[s * cw + c0], fq[s * cw + c0]});
            part_m[(int64_t)blockIdx.x * F + col] = a.m;
            part_q[(int64_t)blockIdx.x * F + col] = a.q;
        }
        __syncthreads();
    }
}

// mean[f], var[f] (biased) from the chunks' pairs.  A block of 1024 threads owns eight columns; its 128 thread
// rows take the chunks round-robin (eight loads in flight each) and are then merged through LDS by a fixed
// halving tree: a short chain of dependent merges instead of one per chunk.
constexpr int kMergeThreads = 1024, kMergeCols = 8, kMergeSlots = kMergeThreads / kMergeCols;

__global__ __launch_bounds__(kMergeThreads) void column_moments_merge_kernel(const float *__restrict__ part_m,
                                                                             const float *__restrict__ part_q,
                                                                             int chunks, int64_t N,
                                                                             int64_t rows_per_chunk, int F,
                                                                             float *__restrict__ mean,
                                                                             float *__restrict__ var)
{
    __shared__ float fn[kMergeSlots][kMergeCols], fm[kMergeSlots][kMergeCols], fq[kMergeSlots][kMergeCols];
    const int c0 = threadIdx.x % kMergeCols, slot = threadIdx.x / kMergeCols;
    const int col = blockIdx.x * kMergeCols + c0;
    const bool ok = col < F;
    const int colc = ok ? col : 0;
    Moments a{0.0f, 0.0f, 0.0f};
    for (int ch0 = slot; ch0 < chunks; ch0 += 8 * kMergeSlots) {   // block-uniform trip count would not matter: no barrier inside
        float pm[8], pq[8], pn[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int ch = min(ch0 + u * kMergeSlots, chunks - 1);
            const int64_t r0 = (int64_t)ch * rows_per_chunk;
            const int64_t cnt = min(N, r0 + rows_per_chunk) - r0;
            pn[u] = (ok && ch0 + u * kMergeSlots < chunks && cnt > 0) ? (float)cnt : 0.0f;
            pm[u] = part_m[(int64_t)ch * F + colc];
            pq[u] = part_q[(int64_t)ch * F + colc];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) moments_merge(a, Moments{pn[u], pm[u], pq[u]});
    }
    fn[slot][c0] = a.n;
    fm[slot][c0] = a.m;
    fq[slot][c0] = a.q;
    __syncthreads();
#pragma unroll
    for (int h = kMergeSlots / 2; h >= 1; h >>= 1) {
        if (slot < h) {
            moments_merge(a, Moments{fn[slot + h][c0], fm[slot + h][c0], fq[slot + h][c0]});
            fn[slot][c0] = a.n;
            fm[slot][c0] = a.m;
            fq[slot][c0] = a.q;
        }
        __syncthreads();
    }
    if (slot == 0 && ok) {
        mean[col] = a.m;
        var[col] = a.q / (float)N;
    }
}

// Few rows (a collated batch of small graphs): one launch for both statistics.  A block of 1024 threads owns
// eight columns; its 128 thread rows take the rows round-robin, several loads in flight each, and are folded
// through LDS by a fixed halving tree; first the mean, then the mean of squared deviations.
constexpr int kSmallRows = 8192;
constexpr int kSmallThreads = 1024, kSmallCols = 8, kSmallSlices = kSmallThreads / kSmallCols;

__device__ __forceinline__ float fold_slices(float (*fold)[kSmallCols], int rs, int c0, float v)
{
    __syncthreads();
    fold[rs][c0] = v;
    __syncthreads();
#pragma unroll
    for (int h = kSmallSlices / 2; h >= 1; h >>= 1) {
        if (rs < h) fold[rs][c0] += fold[rs + h][c0];
        __syncthreads();
    }
    return fold[0][c0];
}

__global__ __launch_bounds__(kSmallThreads) void small_column_stats_kernel(const float *__restrict__ x, int N, int F,
                                                                           float *__restrict__ mean,
                                                                           float *__restrict__ var)
{
    __shared__ float fold[kSmallSlices][kSmallCols];
    const int c0 = threadIdx.x % kSmallCols, rs = threadIdx.x / kSmallCols;
    const int col = blockIdx.x * kSmallCols + c0;
    const bool ok = col < F;
    const float *xc = x + (ok ? col : 0);
    float s = 0.0f;
    if (ok) {
#pragma unroll 8
        for (int row = rs; row < N; row += kSmallSlices) s += xc[(int64_t)row * F];
    }
    const float mu = fold_slices(fold, rs, c0, s) / (float)N;
    float q = 0.0f;
    if (ok) {
#pragma unroll 8
        for (int row = rs; row < N; row += kSmallSlices) {
            const float d = xc[(int64_t)row * F] - mu;
            q = fmaf(d, d, q);
        }
    }
    const float ss = fold_slices(fold, rs, c0, q);
    if (rs == 0 && ok) {
        mean[col] = mu;
        var[col] = ss / (float)N;
    }
}

// out = act(gamma * (x - mean) / sqrt(var + eps) + beta)
__global__ __launch_bounds__(kThreads) void normalise_rows_kernel(const float *__restrict__ x, int64_t N, int F,
                                                                  const float *__restrict__ mean,
                                                                  const float *__restrict__ var,
                                                                  const float *__restrict__ gamma,
                                                                  const float *__restrict__ beta, float eps, int relu,
                                                                  float *__restrict__ out)
{
    const int64_t total = N * F;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total; idx += stride) {
        const int f = (int)(idx % F);
        const float inv = 1.0f / sqrtf(var[f] + eps);
        float y = (gamma ? gamma[f] : 1.0f) * ((x[idx] - mean[f]) * inv) + (beta ? beta[f] : 0.0f);
        if (relu) y = fmaxf(y, 0.0f);
        out[idx] = y;
    }
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

struct ChainLayout {
    size_t h1, h2, h3, pooled, stats, gcn, bn, total;
};

ChainLayout chain_layout(int64_t N, int G, int f1, int f2)
{
    ChainLayout l{};
    l.h1 = 0;
    l.h2 = l.h1 + align256((size_t)N * f1 * sizeof(float));
    l.h3 = l.h2 + align256((size_t)N * f1 * sizeof(float));
    l.pooled = l.h3 + align256((size_t)N * f2 * sizeof(float));
    l.stats = l.pooled + align256((size_t)G * f2 * sizeof(float));
    l.gcn = l.stats + align256((size_t)2 * f1 * sizeof(float));
    l.bn = l.gcn + align256(gnn_gcnconv_workspace_bytes((int32_t)N, std::max(f1, f2)));
    l.total = l.bn + align256(gnn_batchnorm_workspace_bytes((int32_t)N, f1));
    return l;
}

// Column means and (biased) variances of x [N x F]: one launch for few rows, else per-chunk moments and their merge.
gnn_status launch_column_moments(const float *d_x, int64_t N, int F, float *d_mean, float *d_var, void *d_workspace,
                                 size_t workspace_bytes, hipStream_t s)
{
    if (N <= kSmallRows) {
        hipLaunchKernelGGL(small_column_stats_kernel, dim3((unsigned)gnn_div_up(F, kSmallCols)), dim3(kSmallThreads), 0, s, d_x, (int)N,
                           F, d_mean, d_var);
        GNN_LAUNCH_CHECK();
        return GNN_OK;
    }
    if (!d_workspace) return GNN_ERR_NULL;
    if (workspace_bytes < gnn_batchnorm_workspace_bytes((int32_t)N, F)) return GNN_ERR_BAD_SIZE;
    const int chunks = gnn_row_chunk_count(N);
    const int64_t rows_per_chunk = gnn_div_up(N, chunks);
    float *part_m = static_cast<float *>(d_workspace), *part_q = part_m + (size_t)chunks * F;
    hipLaunchKernelGGL(column_moments_partial_kernel, dim3((unsigned)chunks), dim3(kThreads), 0, s, d_x, N, F,
                       rows_per_chunk, part_m, part_q);
    GNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(column_moments_merge_kernel, dim3((unsigned)gnn_div_up(F, kMergeCols)), dim3(kMergeThreads), 0,
                       s, part_m, part_q, chunks, N, rows_per_chunk, F, d_mean, d_var);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

}  // namespace

extern "C" {

size_t gnn_batchnorm_workspace_bytes(int32_t num_rows, int32_t feat_dim)
{
    if (num_rows <= 0 || feat_dim <= 0) return 0;
    return align256(2 * (size_t)gnn_row_chunk_count(num_rows) * feat_dim * sizeof(float));   // (mean, M2) per chunk
}

gnn_status gnn_batchnorm(const float *d_x, int32_t num_rows, int32_t feat_dim, const float *d_gamma,
                         const float *d_beta, float eps, gnn_activation act, int32_t use_given_stats,
                         float *d_mean, float *d_var, float *d_out, void *d_workspace, size_t workspace_bytes,
                         void *stream)
{
    if (!d_x || !d_out || !d_mean || !d_var) return GNN_ERR_NULL;
    if (num_rows <= 0 || feat_dim <= 0 || !(eps >= 0.0f)) return GNN_ERR_BAD_SIZE;
    if (act != GNN_ACT_NONE && act != GNN_ACT_RELU) return GNN_ERR_BAD_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t N = num_rows;
    const int F = feat_dim;
    if (!use_given_stats) GNN_TRY(launch_column_moments(d_x, N, F, d_mean, d_var, d_workspace, workspace_bytes, s));
    const int blocks = (int)std::min<int64_t>(gnn_div_up(N * F, kThreads), 256 * 64);
    hipLaunchKernelGGL(normalise_rows_kernel, dim3(blocks), dim3(kThreads), 0, s, d_x, N, F, d_mean, d_var, d_gamma,
                       d_beta, eps, act == GNN_ACT_RELU ? 1 : 0, d_out);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_dense(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n, const float *d_bias,
                     gnn_activation act, float *d_out, void *stream)
{
    if (act != GNN_ACT_NONE && act != GNN_ACT_RELU) return GNN_ERR_BAD_SIZE;
    // bias and activation ride in the product's store
    GNN_TRY(gnn_launch_xw(d_x, rows, k, d_w, n, nullptr, d_bias, act == GNN_ACT_RELU, d_out,
                          static_cast<hipStream_t>(stream)));
    return GNN_OK;
}

size_t gnn_example_model_workspace_bytes(int32_t num_nodes, int32_t num_graphs, int32_t f1, int32_t f2)
{
    if (num_nodes <= 0 || num_graphs <= 0 || f1 <= 0 || f2 <= 0) return 0;
    return chain_layout(num_nodes, num_graphs, f1, f2).total;
}

gnn_status gnn_example_model_forward(const gnn_graph *g, const int32_t *d_graph_indicator, int32_t num_graphs,
                                     const float *d_x, int32_t f0, const float *d_w1, const float *d_b1, int32_t f1,
                                     const float *d_gamma, const float *d_beta, float eps, const float *d_w2,
                                     const float *d_b2, int32_t f2, const float *d_w3, const float *d_b3, int32_t f3,
                                     float *d_y, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!g || !d_graph_indicator || !d_x || !d_w1 || !d_w2 || !d_w3 || !d_y || !d_workspace) return GNN_ERR_NULL;
    if (num_graphs <= 0 || f0 <= 0 || f1 <= 0 || f2 <= 0 || f3 <= 0) return GNN_ERR_BAD_SIZE;
    const int32_t N = g->num_nodes;
    const ChainLayout l = chain_layout(N, num_graphs, f1, f2);
    if (workspace_bytes < l.total) return GNN_ERR_BAD_SIZE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255u) return GNN_ERR_BAD_SIZE;
    char *ws = static_cast<char *>(d_workspace);
    float *h1 = reinterpret_cast<float *>(ws + l.h1), *h2 = reinterpret_cast<float *>(ws + l.h2),
          *h3 = reinterpret_cast<float *>(ws + l.h3), *pooled = reinterpret_cast<float *>(ws + l.pooled),
          *mean = reinterpret_cast<float *>(ws + l.stats), *var = mean + f1;
    void *gcn_ws = ws + l.gcn, *bn_ws = ws + l.bn;
    const size_t gcn_bytes = l.bn - l.gcn, bn_bytes = l.total - l.bn;

    GNN_TRY(gnn_gcnconv(g, d_x, f0, d_w1, d_b1, f1, 1, GNN_ACT_NONE, h1, gcn_ws, gcn_bytes, stream));
    if (gnn_gcnconv_takes_column_norm(g, h1, f1, d_w2, f2) && eps >= 0.0f) {
        // The normalised activations are never written: the second convolution's projection normalises the rows
        // of h1 as it reads them (the statistics need their own pass over h1 first).
        GNN_TRY(launch_column_moments(h1, N, f1, mean, var, bn_ws, bn_bytes, static_cast<hipStream_t>(stream)));
        gnn_column_norm norm;
        norm.mean = mean; norm.var = var; norm.gamma = d_gamma; norm.beta = d_beta; norm.eps = eps; norm.relu = 1;
        GNN_TRY(gnn_launch_gcnconv(g, h1, f1, d_w2, d_b2, f2, 1, GNN_ACT_RELU, h3, gcn_ws, gcn_bytes, stream, &norm));
    } else {
        GNN_TRY(gnn_batchnorm(h1, N, f1, d_gamma, d_beta, eps, GNN_ACT_RELU, 0, mean, var, h2, bn_ws, bn_bytes, stream));
        GNN_TRY(gnn_gcnconv(g, h2, f1, d_w2, d_b2, f2, 1, GNN_ACT_RELU, h3, gcn_ws, gcn_bytes, stream));
    }
    GNN_TRY(gnn_graph_pool(d_graph_indicator, N, num_graphs, h3, f2, GNN_AGGR_MEAN, pooled, stream));
    return gnn_dense(pooled, num_graphs, f2, d_w3, f3, d_b3, GNN_ACT_NONE, d_y, stream);
}

}  // extern "C"
