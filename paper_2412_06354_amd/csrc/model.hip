// The dense-side layers of the paper's example model (section 3, "Training Example":
// GNNChain(GCNConv(16 => 64), BatchNorm(64), relu, GCNConv(64 => 64, relu), GlobalPool(mean),
// Dense(64, 1))) and the chain itself as one call:
//   * batch normalisation across the node dimension, with batch statistics (two passes: mean, then the
//     mean of squared deviations -- no cancellation) or stored ones, optional relu fused;
//   * a dense layer act(X W + b) on the MFMA projection kernel;
//   * the forward chain, which only sequences entry points of this library on the caller's stream.
// Column statistics use the two-stage scheme of the backward passes: per-chunk partial sums,
// then a fixed-order sum over chunks (deterministic, no atomics).
#include "gnn_internal.h"

#include <algorithm>

namespace {

constexpr int kThreads = 256;

// partial[chunk][f] = sum over the chunk's rows of (x[row,f] - centre[f])^POW   (centre may be NULL = 0)
template <int POW>
__global__ __launch_bounds__(kThreads) void column_moment_partial_kernel(const float *__restrict__ x, int64_t N,
                                                                         int F, const float *__restrict__ centre,
                                                                         int64_t rows_per_chunk,
                                                                         float *__restrict__ partial)
{
    __shared__ float fold[kThreads];
    const int cw = min(F, kThreads), slices = kThreads / cw;
    const int rs = threadIdx.x / cw, c0 = threadIdx.x % cw;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk, r1 = min(N, r0 + rows_per_chunk);
    for (int cbase = 0; cbase < F; cbase += cw) {
        const int col = cbase + c0;
        float s[2] = {0.0f, 0.0f};   // two interleaved running sums
        if (rs < slices && col < F) {
            const float mu = centre ? centre[col] : 0.0f;
            int64_t row = r0 + rs;
            for (; row + slices < r1; row += 2 * slices) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const float d = x[(row + u * slices) * F + col] - mu;
                    s[u] += POW == 2 ? d * d : d;
                }
            }
            if (row < r1) {
                const float d = x[row * F + col] - mu;
                s[0] += POW == 2 ? d * d : d;
            }
        }
        fold[threadIdx.x] = s[0] + s[1];
        __syncthreads();
        if (rs == 0 && col < F) {
            float t = 0.0f;
            for (int q = 0; q < slices; ++q) t += fold[q * cw + c0];
            partial[(int64_t)blockIdx.x * F + col] = t;
        }
        __syncthreads();
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

}  // namespace

extern "C" {

size_t gnn_batchnorm_workspace_bytes(int32_t num_rows, int32_t feat_dim)
{
    if (num_rows <= 0 || feat_dim <= 0) return 0;
    return align256((size_t)gnn_row_chunk_count(num_rows) * feat_dim * sizeof(float));
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
    if (!use_given_stats && N <= kSmallRows) {
        hipLaunchKernelGGL(small_column_stats_kernel, dim3((unsigned)gnn_div_up(F, kSmallCols)), dim3(kSmallThreads), 0, s, d_x, (int)N,
                           F, d_mean, d_var);
        GNN_LAUNCH_CHECK();
    } else if (!use_given_stats) {
        if (!d_workspace) return GNN_ERR_NULL;
        if (workspace_bytes < gnn_batchnorm_workspace_bytes(num_rows, feat_dim)) return GNN_ERR_BAD_SIZE;
        float *part = static_cast<float *>(d_workspace);
        const int chunks = gnn_row_chunk_count(N);
        const int64_t rows_per_chunk = gnn_div_up(N, chunks);
        hipLaunchKernelGGL(column_moment_partial_kernel<1>, dim3((unsigned)chunks), dim3(kThreads), 0, s, d_x, N, F,
                           (const float *)nullptr, rows_per_chunk, part);
        GNN_LAUNCH_CHECK();
        GNN_TRY(gnn_launch_sum_partials_scaled(part, chunks, F, 1.0f / (float)N, d_mean, s));
        hipLaunchKernelGGL(column_moment_partial_kernel<2>, dim3((unsigned)chunks), dim3(kThreads), 0, s, d_x, N, F,
                           (const float *)d_mean, rows_per_chunk, part);
        GNN_LAUNCH_CHECK();
        GNN_TRY(gnn_launch_sum_partials_scaled(part, chunks, F, 1.0f / (float)N, d_var, s));
    }
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
    GNN_TRY(gnn_batchnorm(h1, N, f1, d_gamma, d_beta, eps, GNN_ACT_RELU, 0, mean, var, h2, bn_ws, bn_bytes, stream));
    GNN_TRY(gnn_gcnconv(g, h2, f1, d_w2, d_b2, f2, 1, GNN_ACT_RELU, h3, gcn_ws, gcn_bytes, stream));
    GNN_TRY(gnn_graph_pool(d_graph_indicator, N, num_graphs, h3, f2, GNN_AGGR_MEAN, pooled, stream));
    return gnn_dense(pooled, num_graphs, f2, d_w3, f3, d_b3, GNN_ACT_NONE, d_y, stream);
}

}  // extern "C"
