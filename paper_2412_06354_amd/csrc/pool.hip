// Graph-level readout of a batch of graphs (GlobalPool in the paper's training example): the
// batch is the block-diagonal union of many small graphs with one graph id per node, ids
// non-decreasing, so every graph is a contiguous run of node rows.
//
// One block per graph: the run's bounds come from two block-wide searches in the sorted ids; the
// block's threads are arranged as (node slot, feature lane), node slots stride over the run and
// are combined through LDS in slot order, so the result does not depend on scheduling.
#include "gnn_internal.h"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float max_pz(float a, float b)
{
    if (a > b) return a;
    if (b > a) return b;
    return __uint_as_float(__float_as_uint(a) & __float_as_uint(b));
}

// First index whose value is >= key in the sorted array a[0..n), found by the whole block: every
// round the 256 threads probe evenly spaced positions of the remaining range and count how many
// are still below the key, which narrows the range 256-fold (a handful of rounds instead of
// log2(n) dependent loads).
__device__ __forceinline__ int block_lower_bound(const int32_t *__restrict__ a, int n, int key)
{
    int lo = 0, hi = n;   // the answer lies in [lo, hi]
    while (lo < hi) {
        const int step = (hi - lo + kThreads - 1) / kThreads;
        const int pos = lo + (int)threadIdx.x * step;
        const int below = (pos < hi) && (a[pos] < key);
        const int c = __syncthreads_count(below);   // the array is sorted: exactly probes 0 .. c-1 are below the key
        if (c == 0) return lo;
        const int new_hi = min(hi, lo + c * step);  // probe c (if inside) is >= key
        lo = lo + (c - 1) * step + 1;               // probe c-1 is below the key
        hi = new_hi;
    }
    return lo;
}

template <bool MAX>
__global__ __launch_bounds__(kThreads) void pool_kernel(const int32_t *__restrict__ gi, int32_t N, const float *__restrict__ x,
                                                        int32_t F, int32_t lanes /* power of two <= 256 */, int mean,
                                                        float *__restrict__ out)
{
    __shared__ float part[kThreads];
    const int g = blockIdx.x;
    const int lo = block_lower_bound(gi, N, g), hi = block_lower_bound(gi, N, g + 1);
    const int fl = threadIdx.x % lanes, slot = threadIdx.x / lanes, slots = kThreads / lanes;
    for (int f0 = 0; f0 < F; f0 += lanes) {
        const int f = f0 + fl;
        float acc = MAX ? -INFINITY : 0.0f;
        if (f < F)
            for (int i = lo + slot; i < hi; i += slots) {
                const float v = x[(int64_t)i * F + f];
                acc = MAX ? max_pz(acc, v) : acc + v;
            }
        part[threadIdx.x] = acc;
        __syncthreads();
        if (slot == 0 && f < F) {
            for (int s = 1; s < slots; ++s) {
                const float v = part[s * lanes + fl];
                acc = MAX ? max_pz(acc, v) : acc + v;
            }
            const int cnt = hi - lo;
            if (cnt == 0) acc = 0.0f;
            if (mean && cnt > 0) acc = acc / (float)cnt;
            out[(int64_t)g * F + f] = acc;
        }
        __syncthreads();
    }
}

// Backward of sum / mean pooling: every node of graph g receives gout[g,:] (divided by the node count for
// the mean).  One block per graph, same run search as the forward kernel; rows are written coalesced.
__global__ __launch_bounds__(kThreads) void pool_backward_kernel(const int32_t *__restrict__ gi, int32_t N,
                                                                 const float *__restrict__ gout, int32_t F, int mean,
                                                                 float *__restrict__ gx)
{
    const int g = blockIdx.x;
    const int lo = block_lower_bound(gi, N, g), hi = block_lower_bound(gi, N, g + 1);
    const int cnt = hi - lo;
    if (cnt <= 0) return;   // block-uniform
    const int64_t total = (int64_t)cnt * F;
    for (int64_t q = threadIdx.x; q < total; q += kThreads) {
        const int f = (int)(q % F);
        const float v = gout[(int64_t)g * F + f];
        gx[(int64_t)lo * F + q] = mean ? v / (float)cnt : v;
    }
}

}  // namespace

extern "C" gnn_status gnn_graph_pool_backward(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                              const float *d_grad_out, int32_t feat_dim, gnn_aggr aggr,
                                              float *d_grad_x, void *stream)
{
    if (num_nodes < 0 || num_graphs <= 0 || feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (aggr == GNN_AGGR_MAX || aggr == GNN_AGGR_MIN || aggr == GNN_AGGR_PROD) return GNN_ERR_UNSUPPORTED;
    if (aggr != GNN_AGGR_SUM && aggr != GNN_AGGR_MEAN) return GNN_ERR_BAD_SIZE;
    if (num_nodes == 0) return GNN_OK;
    if (!d_graph_indicator || !d_grad_out || !d_grad_x) return GNN_ERR_NULL;
    hipLaunchKernelGGL(pool_backward_kernel, dim3((unsigned)num_graphs), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), d_graph_indicator, num_nodes, d_grad_out, feat_dim,
                       aggr == GNN_AGGR_MEAN ? 1 : 0, d_grad_x);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

extern "C" gnn_status gnn_graph_pool(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                     const float *d_x, int32_t feat_dim, gnn_aggr aggr, float *d_out, void *stream)
{
    if (!d_out) return GNN_ERR_NULL;
    if (num_nodes < 0 || num_graphs <= 0 || feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (aggr != GNN_AGGR_SUM && aggr != GNN_AGGR_MEAN && aggr != GNN_AGGR_MAX) return GNN_ERR_BAD_SIZE;
    if (num_nodes > 0 && (!d_graph_indicator || !d_x)) return GNN_ERR_NULL;
    int lanes = 1;
    while (lanes < feat_dim && lanes < kThreads) lanes <<= 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (aggr == GNN_AGGR_MAX)
        hipLaunchKernelGGL(pool_kernel<true>, dim3((unsigned)num_graphs), dim3(kThreads), 0, s, d_graph_indicator,
                           num_nodes, d_x, feat_dim, lanes, 0, d_out);
    else
        hipLaunchKernelGGL(pool_kernel<false>, dim3((unsigned)num_graphs), dim3(kThreads), 0, s, d_graph_indicator,
                           num_nodes, d_x, feat_dim, lanes, aggr == GNN_AGGR_MEAN ? 1 : 0, d_out);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}
