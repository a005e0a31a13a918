// Training-side pieces of the paper's example (section 3, "Training Example": mean-squared-error loss,
// reverse-mode gradients of the whole chain, Adam(1e-4) update): backward of the dense layer and of the
// batch normalisation (optionally through the relu that followed it), a relu mask, the loss gradient,
// the Adam step, and one training step of the example model as a single call that only sequences
// entry points of this library on the caller's stream.  All reductions are two-stage with a fixed
// order (no atomics): a training step is bitwise reproducible.
#include "gnn_internal.h"

#include <algorithm>
#include <cmath>

namespace {

constexpr int kThreads = 256;

// loss = mean (pred - target)^2,  grad = 2 (pred - target) / count.  One block; fixed summation order.
__global__ __launch_bounds__(kThreads) void mse_kernel(const float *__restrict__ pred, const float *__restrict__ target,
                                                       int64_t count, float *__restrict__ loss,
                                                       float *__restrict__ grad)
{
    __shared__ float fold[kThreads];
    float s = 0.0f;
    const float inv = 1.0f / (float)count;
    for (int64_t i = threadIdx.x; i < count; i += kThreads) {
        const float d = pred[i] - target[i];
        s = fmaf(d, d, s);
        if (grad) grad[i] = 2.0f * d * inv;
    }
    fold[threadIdx.x] = s;
    __syncthreads();
    for (int off = kThreads / 2; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) fold[threadIdx.x] += fold[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0 && loss) *loss = fold[0] * inv;
}

// gx = y > 0 ? gy : 0   (gx may alias gy)
__global__ __launch_bounds__(kThreads) void relu_mask_kernel(const float *__restrict__ y, const float *gy, int64_t n,
                                                             float *gx)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) gx[i] = y[i] > 0.0f ? gy[i] : 0.0f;
}

// Batch-norm backward, stage 1: per row chunk and column, sum of g and of g * xhat, where
// g = gy masked by (y > 0) when y is given (the relu that followed) and xhat = (x - mean) / sqrt(var + eps).
template <bool MASK>
__global__ __launch_bounds__(kThreads) void bn_backward_partial_kernel(const float *__restrict__ x, int64_t N, int F,
                                                                       const float *__restrict__ mean,
                                                                       const float *__restrict__ var, float eps,
                                                                       const float *__restrict__ gy,
                                                                       const float *__restrict__ y,
                                                                       int64_t rows_per_chunk,
                                                                       float *__restrict__ part_b,
                                                                       float *__restrict__ part_g)
{
    __shared__ float fold_b[kThreads], fold_g[kThreads];
    const int cw = min(F, kThreads), slices = kThreads / cw;
    const int rs = threadIdx.x / cw, c0 = threadIdx.x % cw;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk, r1 = min(N, r0 + rows_per_chunk);
    for (int cbase = 0; cbase < F; cbase += cw) {
        const int col = cbase + c0;
        float sb = 0.0f, sg = 0.0f;
        if (rs < slices && col < F) {
            const float mu = mean[col], inv = 1.0f / sqrtf(var[col] + eps);
            // four rows per round, all loads first (no branch in the body: the mask is a template parameter)
            int64_t row = r0 + rs;
            for (; row + 3 * slices < r1; row += 4 * slices) {
                float gv[4], xv[4], yv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t q = (row + u * slices) * F + col;
                    gv[u] = gy[q];
                    xv[u] = x[q];
                    yv[u] = MASK ? y[q] : 1.0f;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float g = yv[u] > 0.0f ? gv[u] : 0.0f;
                    sb += g;
                    sg = fmaf(g, (xv[u] - mu) * inv, sg);
                }
            }
            for (; row < r1; row += slices) {
                const int64_t q = row * F + col;
                float g = gy[q];
                if (MASK) g = y[q] > 0.0f ? g : 0.0f;
                sb += g;
                sg = fmaf(g, (x[q] - mu) * inv, sg);
            }
        }
        fold_b[threadIdx.x] = sb;
        fold_g[threadIdx.x] = sg;
        __syncthreads();
        if (rs == 0 && col < F) {
            float tb = 0.0f, tg = 0.0f;
            for (int q = 0; q < slices; ++q) {
                tb += fold_b[q * cw + c0];
                tg += fold_g[q * cw + c0];
            }
            part_b[(int64_t)blockIdx.x * F + col] = tb;
            part_g[(int64_t)blockIdx.x * F + col] = tg;
        }
        __syncthreads();
    }
}

// Few rows: both column sums in one launch.  A block of 1024 threads owns eight columns; its 128 thread rows
// take the rows round-robin and are folded through LDS by a fixed halving tree.
constexpr int kSmallRows = 8192;
constexpr int kSmallThreads = 1024, kSmallCols = 8, kSmallSlices = kSmallThreads / kSmallCols;

__global__ __launch_bounds__(kSmallThreads) void small_bn_backward_sums_kernel(
    const float *__restrict__ x, int N, int F, const float *__restrict__ mean, const float *__restrict__ var, float eps,
    const float *__restrict__ gy, const float *__restrict__ y, float *__restrict__ gbeta, float *__restrict__ ggamma)
{
    __shared__ float fold_b[kSmallSlices][kSmallCols], fold_g[kSmallSlices][kSmallCols];
    const int c0 = threadIdx.x % kSmallCols, rs = threadIdx.x / kSmallCols;
    const int col = blockIdx.x * kSmallCols + c0;
    const bool ok = col < F;
    float sb = 0.0f, sg = 0.0f;
    if (ok) {
        const float mu = mean[col], inv = 1.0f / sqrtf(var[col] + eps);
#pragma unroll 4
        for (int row = rs; row < N; row += kSmallSlices) {
            const int64_t q = (int64_t)row * F + col;
            float g = gy[q];
            if (y) g = y[q] > 0.0f ? g : 0.0f;
            sb += g;
            sg = fmaf(g, (x[q] - mu) * inv, sg);
        }
    }
    fold_b[rs][c0] = sb;
    fold_g[rs][c0] = sg;
    __syncthreads();
#pragma unroll
    for (int h = kSmallSlices / 2; h >= 1; h >>= 1) {
        if (rs < h) {
            fold_b[rs][c0] += fold_b[rs + h][c0];
            fold_g[rs][c0] += fold_g[rs + h][c0];
        }
        __syncthreads();
    }
    if (rs == 0 && ok) {
        gbeta[col] = fold_b[0][c0];
        ggamma[col] = fold_g[0][c0];
    }
}

// stage 2: gx = gamma * inv * (g - gbeta / N - xhat * ggamma / N)
__global__ __launch_bounds__(kThreads) void bn_backward_apply_kernel(const float *__restrict__ x, int64_t N, int F,
                                                                     const float *__restrict__ mean,
                                                                     const float *__restrict__ var, float eps,
                                                                     const float *__restrict__ gamma,
                                                                     const float *gy, const float *__restrict__ y,
                                                                     const float *__restrict__ gbeta,
                                                                     const float *__restrict__ ggamma, float *gx)
{
    const int64_t total = N * F;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    const float inv_n = 1.0f / (float)N;
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total; idx += stride) {
        const int f = (int)(idx % F);
        const float inv = 1.0f / sqrtf(var[f] + eps);
        const float xh = (x[idx] - mean[f]) * inv;
        float g = gy[idx];
        if (y) g = y[idx] > 0.0f ? g : 0.0f;
        gx[idx] = (gamma ? gamma[f] : 1.0f) * inv * (g - gbeta[f] * inv_n - xh * ggamma[f] * inv_n);
    }
}

// column sums, stage 1 (stage 2 is gnn_launch_sum_partials)
__global__ __launch_bounds__(kThreads) void column_sum_partial_kernel(const float *__restrict__ g, int64_t N, int F,
                                                                      int64_t rows_per_chunk,
                                                                      float *__restrict__ partial)
{
    __shared__ float fold[kThreads];
    const int cw = min(F, kThreads), slices = kThreads / cw;
    const int rs = threadIdx.x / cw, c0 = threadIdx.x % cw;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk, r1 = min(N, r0 + rows_per_chunk);
    for (int cbase = 0; cbase < F; cbase += cw) {
        const int col = cbase + c0;
        float s = 0.0f;
        if (rs < slices && col < F)
            for (int64_t row = r0 + rs; row < r1; row += slices) s += g[row * F + col];
        fold[threadIdx.x] = s;
        __syncthreads();
        if (rs == 0 && col < F) {
            float t = 0.0f;
            for (int q = 0; q < slices; ++q) t += fold[q * cw + c0];
            partial[(int64_t)blockIdx.x * F + col] = t;
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(kThreads) void adam_kernel(float *__restrict__ p, float *__restrict__ m,
                                                        float *__restrict__ v, const float *__restrict__ g, int64_t n,
                                                        float lr, float b1, float b2, float eps, float c1, float c2)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const float gi = g[i];
        const float mi = b1 * m[i] + (1.0f - b1) * gi;
        const float vi = b2 * v[i] + (1.0f - b2) * gi * gi;
        m[i] = mi;
        v[i] = vi;
        p[i] = p[i] - lr * (mi / c1) / (sqrtf(vi / c2) + eps);
    }
}

// The eight parameter arrays of the example model in one launch (blockIdx.y = which array).
struct AdamBatch {
    float *p[8], *m[8], *v[8];
    const float *g[8];
    int64_t n[8];
};

__global__ __launch_bounds__(kThreads) void adam_batch_kernel(const AdamBatch b, float lr, float b1, float b2, float eps,
                                                              float c1, float c2)
{
    const int a = blockIdx.y;
    float *p = b.p[a], *m = b.m[a], *v = b.v[a];
    const float *g = b.g[a];
    const int64_t n = b.n[a];
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const float gi = g[i];
        const float mi = b1 * m[i] + (1.0f - b1) * gi;
        const float vi = b2 * v[i] + (1.0f - b2) * gi * gi;
        m[i] = mi;
        v[i] = vi;
        p[i] = p[i] - lr * (mi / c1) / (sqrtf(vi / c2) + eps);
    }
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

int grid_for(int64_t n) { return (int)std::max<int64_t>(1, std::min<int64_t>(gnn_div_up(n, kThreads), 256 * 64)); }

struct StepLayout {
    size_t h1, h2, h3, pooled, y, stats, gy, gpooled, gh3, gh2, gh1, pgrad, gcn_f, gcn_b, bn, dense_b, total;
    size_t pg_off[8];   // floats, relative to pgrad
};

StepLayout step_layout(int64_t N, int G, int f0, int f1, int f2, int f3)
{
    StepLayout l{};
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o += align256(bytes); return r; };
    const size_t F4 = sizeof(float);
    l.h1 = take((size_t)N * f1 * F4);
    l.h2 = take((size_t)N * f1 * F4);
    l.h3 = take((size_t)N * f2 * F4);
    l.pooled = take((size_t)G * f2 * F4);
    l.y = take((size_t)G * f3 * F4);
    l.stats = take((size_t)2 * f1 * F4);
    l.gy = take((size_t)G * f3 * F4);
    l.gpooled = take((size_t)G * f2 * F4);
    l.gh3 = take((size_t)N * f2 * F4);
    l.gh2 = take((size_t)N * f1 * F4);
    l.gh1 = take((size_t)N * f1 * F4);
    const size_t sizes[8] = {(size_t)f0 * f1, (size_t)f1, (size_t)f1, (size_t)f1,
                             (size_t)f1 * f2, (size_t)f2, (size_t)f2 * f3, (size_t)f3};
    size_t pf = 0;
    for (int q = 0; q < 8; ++q) {
        l.pg_off[q] = pf;
        pf += (sizes[q] + 63) & ~(size_t)63;
    }
    l.pgrad = take(pf * F4);
    l.gcn_f = take(gnn_gcnconv_workspace_bytes((int32_t)N, std::max(f1, f2)));
    l.gcn_b = take(std::max(gnn_gcnconv_backward_workspace_bytes((int32_t)N, f0, f1),
                            gnn_gcnconv_backward_workspace_bytes((int32_t)N, f1, f2)));
    l.bn = take(std::max(gnn_batchnorm_workspace_bytes((int32_t)N, f1),
                         gnn_batchnorm_backward_workspace_bytes((int32_t)N, f1)));
    l.dense_b = take(gnn_dense_backward_workspace_bytes(G, f2, f3));
    l.total = o;
    return l;
}

}  // namespace

extern "C" {

gnn_status gnn_mse_loss(const float *d_pred, const float *d_target, int64_t count, float *d_loss, float *d_grad,
                        void *stream)
{
    if (count <= 0) return GNN_ERR_BAD_SIZE;
    if (!d_pred || !d_target || (!d_loss && !d_grad)) return GNN_ERR_NULL;
    hipLaunchKernelGGL(mse_kernel, dim3(1), dim3(kThreads), 0, static_cast<hipStream_t>(stream), d_pred, d_target, count,
                       d_loss, d_grad);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_relu_backward(const float *d_y, const float *d_grad_y, int64_t count, float *d_grad_x, void *stream)
{
    if (count < 0) return GNN_ERR_BAD_SIZE;
    if (count == 0) return GNN_OK;
    if (!d_y || !d_grad_y || !d_grad_x) return GNN_ERR_NULL;
    hipLaunchKernelGGL(relu_mask_kernel, dim3(grid_for(count)), dim3(kThreads), 0, static_cast<hipStream_t>(stream), d_y,
                       d_grad_y, count, d_grad_x);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

size_t gnn_batchnorm_backward_workspace_bytes(int32_t num_rows, int32_t feat_dim)
{
    if (num_rows <= 0 || feat_dim <= 0) return 0;
    return 2 * align256((size_t)gnn_row_chunk_count(num_rows) * feat_dim * sizeof(float));
}

gnn_status gnn_batchnorm_backward(const float *d_x, int32_t num_rows, int32_t feat_dim, const float *d_gamma,
                                  const float *d_mean, const float *d_var, float eps, const float *d_grad_y,
                                  const float *d_y_relu, float *d_grad_x, float *d_grad_gamma, float *d_grad_beta,
                                  void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!d_x || !d_mean || !d_var || !d_grad_y || !d_grad_gamma || !d_grad_beta || !d_workspace) return GNN_ERR_NULL;
    if (num_rows <= 0 || feat_dim <= 0 || !(eps >= 0.0f)) return GNN_ERR_BAD_SIZE;
    if (workspace_bytes < gnn_batchnorm_backward_workspace_bytes(num_rows, feat_dim)) return GNN_ERR_BAD_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t N = num_rows;
    const int F = feat_dim;
    const int chunks = gnn_row_chunk_count(N);
    const int64_t rows_per_chunk = gnn_div_up(N, chunks);
    float *part_b = static_cast<float *>(d_workspace);
    float *part_g = reinterpret_cast<float *>(static_cast<char *>(d_workspace) +
                                              align256((size_t)chunks * F * sizeof(float)));
    if (N <= kSmallRows) {
        hipLaunchKernelGGL(small_bn_backward_sums_kernel, dim3((unsigned)gnn_div_up(F, kSmallCols)),
                           dim3(kSmallThreads), 0, s, d_x,
                           (int)N, F, d_mean, d_var, eps, d_grad_y, d_y_relu, d_grad_beta, d_grad_gamma);
        GNN_LAUNCH_CHECK();
    } else {
        if (d_y_relu)
            hipLaunchKernelGGL(bn_backward_partial_kernel<true>, dim3((unsigned)chunks), dim3(kThreads), 0, s, d_x, N, F,
                               d_mean, d_var, eps, d_grad_y, d_y_relu, rows_per_chunk, part_b, part_g);
        else
            hipLaunchKernelGGL(bn_backward_partial_kernel<false>, dim3((unsigned)chunks), dim3(kThreads), 0, s, d_x, N, F,
                               d_mean, d_var, eps, d_grad_y, d_y_relu, rows_per_chunk, part_b, part_g);
        GNN_LAUNCH_CHECK();
        GNN_TRY(gnn_launch_sum_partials(part_b, chunks, F, d_grad_beta, s));
        GNN_TRY(gnn_launch_sum_partials(part_g, chunks, F, d_grad_gamma, s));
    }
    if (d_grad_x) {
        hipLaunchKernelGGL(bn_backward_apply_kernel, dim3(grid_for(N * F)), dim3(kThreads), 0, s, d_x, N, F, d_mean,
                           d_var, eps, d_gamma, d_grad_y, d_y_relu, d_grad_beta, d_grad_gamma, d_grad_x);
        GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
}

size_t gnn_dense_backward_workspace_bytes(int64_t rows, int32_t k, int32_t n)
{
    if (rows <= 0 || k <= 0 || n <= 0) return 0;
    return align256((size_t)k * n * sizeof(float)) +
           align256((size_t)gnn_row_chunk_count(rows) * std::max(k, 1) * n * sizeof(float));
}

gnn_status gnn_dense_backward(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                              const float *d_grad_y, float *d_grad_x, float *d_grad_w, float *d_grad_b,
                              void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (rows <= 0 || k <= 0 || n <= 0) return GNN_ERR_BAD_SIZE;
    if (!d_grad_y || !d_workspace || (d_grad_x && !d_w) || (d_grad_w && !d_x)) return GNN_ERR_NULL;
    if (workspace_bytes < gnn_dense_backward_workspace_bytes(rows, k, n)) return GNN_ERR_BAD_SIZE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255u) return GNN_ERR_BAD_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *wt = static_cast<float *>(d_workspace);
    float *part = reinterpret_cast<float *>(static_cast<char *>(d_workspace) + align256((size_t)k * n * sizeof(float)));
    if (d_grad_x) {
        GNN_TRY(gnn_launch_transpose(d_w, k, n, wt, s));
        GNN_TRY(gnn_dense_xw(d_grad_y, rows, n, wt, k, nullptr, d_grad_x, stream));
    }
    if (d_grad_w) GNN_TRY(gnn_launch_xty(d_x, d_grad_y, rows, k, n, part, d_grad_w, s));
    if (d_grad_b) {
        const int chunks = gnn_row_chunk_count(rows);
        hipLaunchKernelGGL(column_sum_partial_kernel, dim3((unsigned)chunks), dim3(kThreads), 0, s, d_grad_y, rows, n,
                           gnn_div_up(rows, chunks), part);
        GNN_LAUNCH_CHECK();
        GNN_TRY(gnn_launch_sum_partials(part, chunks, n, d_grad_b, s));
    }
    return GNN_OK;
}

gnn_status gnn_adam_step(float *d_param, float *d_m, float *d_v, const float *d_grad, int64_t count, float lr,
                         float beta1, float beta2, float eps, int32_t step, void *stream)
{
    if (count < 0 || step <= 0) return GNN_ERR_BAD_SIZE;
    if (count == 0) return GNN_OK;
    if (!d_param || !d_m || !d_v || !d_grad) return GNN_ERR_NULL;
    const float c1 = (float)(1.0 - std::pow((double)beta1, (double)step));
    const float c2 = (float)(1.0 - std::pow((double)beta2, (double)step));
    hipLaunchKernelGGL(adam_kernel, dim3(grid_for(count)), dim3(kThreads), 0, static_cast<hipStream_t>(stream), d_param,
                       d_m, d_v, d_grad, count, lr, beta1, beta2, eps, c1, c2);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

size_t gnn_example_model_train_workspace_bytes(int32_t num_nodes, int32_t num_graphs, int32_t f0, int32_t f1,
                                               int32_t f2, int32_t f3)
{
    if (num_nodes <= 0 || num_graphs <= 0 || f0 <= 0 || f1 <= 0 || f2 <= 0 || f3 <= 0) return 0;
    return step_layout(num_nodes, num_graphs, f0, f1, f2, f3).total;
}

gnn_status gnn_example_model_train_step(const gnn_graph *g, const gnn_graph *g_by_source,
                                        const int32_t *d_graph_indicator, int32_t num_graphs, const float *d_x,
                                        int32_t f0, int32_t f1, int32_t f2, int32_t f3, const float *d_target,
                                        float *const *d_params, float *const *d_adam_m, float *const *d_adam_v,
                                        float bn_eps, float lr, float beta1, float beta2, float adam_eps, int32_t step,
                                        float *d_loss, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!g || !g_by_source || !d_graph_indicator || !d_x || !d_target || !d_params || !d_adam_m || !d_adam_v ||
        !d_workspace)
        return GNN_ERR_NULL;
    if (num_graphs <= 0 || f0 <= 0 || f1 <= 0 || f2 <= 0 || f3 <= 0 || step <= 0) return GNN_ERR_BAD_SIZE;
    for (int q = 0; q < 8; ++q)
        if (!d_params[q] || !d_adam_m[q] || !d_adam_v[q]) return GNN_ERR_NULL;
    const int32_t N = g->num_nodes;
    const StepLayout l = step_layout(N, num_graphs, f0, f1, f2, f3);
    if (workspace_bytes < l.total) return GNN_ERR_BAD_SIZE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255u) return GNN_ERR_BAD_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(d_workspace);
    auto at = [&](size_t off) { return reinterpret_cast<float *>(ws + off); };
    float *h1 = at(l.h1), *h2 = at(l.h2), *h3 = at(l.h3), *pooled = at(l.pooled), *y = at(l.y), *mean = at(l.stats),
          *var = mean + f1, *gy = at(l.gy), *gpooled = at(l.gpooled), *gh3 = at(l.gh3), *gh2 = at(l.gh2),
          *gh1 = at(l.gh1), *pg = at(l.pgrad);
    float *w1 = d_params[0], *b1 = d_params[1], *gamma = d_params[2], *beta = d_params[3], *w2 = d_params[4],
          *b2 = d_params[5], *w3 = d_params[6], *b3 = d_params[7];
    float *gw1 = pg + l.pg_off[0], *gb1 = pg + l.pg_off[1], *ggamma = pg + l.pg_off[2], *gbeta = pg + l.pg_off[3],
          *gw2 = pg + l.pg_off[4], *gb2 = pg + l.pg_off[5], *gw3 = pg + l.pg_off[6], *gb3 = pg + l.pg_off[7];
    void *gcn_f = ws + l.gcn_f, *gcn_b = ws + l.gcn_b, *bn = ws + l.bn, *dense_b = ws + l.dense_b;
    const size_t gcn_f_bytes = l.gcn_b - l.gcn_f, gcn_b_bytes = l.bn - l.gcn_b, bn_bytes = l.dense_b - l.bn,
                 dense_b_bytes = l.total - l.dense_b;

    // forward, keeping what the backward pass needs
    GNN_TRY(gnn_gcnconv(g, d_x, f0, w1, b1, f1, 1, GNN_ACT_NONE, h1, gcn_f, gcn_f_bytes, stream));
    GNN_TRY(gnn_batchnorm(h1, N, f1, gamma, beta, bn_eps, GNN_ACT_RELU, 0, mean, var, h2, bn, bn_bytes, stream));
    GNN_TRY(gnn_gcnconv(g, h2, f1, w2, b2, f2, 1, GNN_ACT_RELU, h3, gcn_f, gcn_f_bytes, stream));
    GNN_TRY(gnn_graph_pool(d_graph_indicator, N, num_graphs, h3, f2, GNN_AGGR_MEAN, pooled, stream));
    GNN_TRY(gnn_dense(pooled, num_graphs, f2, w3, f3, b3, GNN_ACT_NONE, y, stream));
    // loss and the chain rule in reverse
    GNN_TRY(gnn_mse_loss(y, d_target, (int64_t)num_graphs * f3, d_loss, gy, stream));
    GNN_TRY(gnn_dense_backward(pooled, num_graphs, f2, w3, f3, gy, gpooled, gw3, gb3, dense_b, dense_b_bytes, stream));
    // pooling backward with the second layer's relu mask in the same pass
    GNN_TRY(gnn_launch_pool_backward(d_graph_indicator, N, num_graphs, gpooled, f2, GNN_AGGR_MEAN, h3, gh3, s));
    GNN_TRY(gnn_gcnconv_backward(g, g_by_source, h2, f1, w2, f2, 1, gh3, gh2, gw2, gb2, gcn_b, gcn_b_bytes, stream));
    GNN_TRY(gnn_batchnorm_backward(h1, N, f1, gamma, mean, var, bn_eps, gh2, h2, gh1, ggamma, gbeta, bn, bn_bytes,
                                   stream));
    GNN_TRY(gnn_gcnconv_backward(g, g_by_source, d_x, f0, w1, f1, 1, gh1, nullptr, gw1, gb1, gcn_b, gcn_b_bytes,
                                 stream));
    // optimiser
    const int64_t counts[8] = {(int64_t)f0 * f1, f1, f1, f1, (int64_t)f1 * f2, f2, (int64_t)f2 * f3, f3};
    AdamBatch batch;
    int64_t largest = 1;
    for (int q = 0; q < 8; ++q) {
        batch.p[q] = d_params[q];
        batch.m[q] = d_adam_m[q];
        batch.v[q] = d_adam_v[q];
        batch.g[q] = pg + l.pg_off[q];
        batch.n[q] = counts[q];
        largest = std::max(largest, counts[q]);
    }
    const float c1 = (float)(1.0 - std::pow((double)beta1, (double)step));
    const float c2 = (float)(1.0 - std::pow((double)beta2, (double)step));
    hipLaunchKernelGGL(adam_batch_kernel, dim3((unsigned)std::min<int64_t>(gnn_div_up(largest, kThreads), 1024), 8),
                       dim3(kThreads), 0, s, batch, lr, beta1, beta2, adam_eps, c1, c2);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

}  // extern "C"
