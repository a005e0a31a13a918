// Graph-level readout of a batch of graphs (GlobalPool in the paper's training example): the
// batch is the block-diagonal union of many small graphs with one graph id per node, ids
// non-decreasing, so every graph is a contiguous run of node rows.
//
// One block per graph: the run's bounds come from two interleaved block-wide searches in the sorted ids; the
// block's threads are arranged as (node slot, feature lane), node slots stride over the run and
// are combined through LDS in slot order, so the result does not depend on scheduling.
#include <algorithm>

#include "gnn_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kSmallGraphNodes = 128;   // average nodes per graph up to which a wavefront takes a graph ...
constexpr int kManyGraphs = 1024;       // ... in batches of at least this many graphs

__device__ __forceinline__ float max_pz(float a, float b)
{
    if (a > b) return a;
    if (b > a) return b;
    return __uint_as_float(__float_as_uint(a) & __float_as_uint(b));   // equal, or the pair (-0, +0): +0
}

// Lower bound (first index whose value is >= key) in the sorted array a[0..n), found by the whole block: every
// round the 256 threads probe evenly spaced positions of the remaining range and count how many are still below
// the key, which narrows the range 256-fold (a handful of rounds instead of log2(n) dependent loads).
// Both ends of graph g's run at once: the lower bounds of g and of g + 1, searched in the same rounds so that
// the two chains of dependent loads overlap (a block spends most of its time in these searches).
__device__ __forceinline__ void block_run_bounds(const int32_t *__restrict__ a, int n, int g, int *first, int *last)
{
    int lo0 = 0, hi0 = n, lo1 = 0, hi1 = n;
    while (lo0 < hi0 || lo1 < hi1) {   // block-uniform
        const int step0 = max(1, (hi0 - lo0 + kThreads - 1) / kThreads), step1 = max(1, (hi1 - lo1 + kThreads - 1) / kThreads);
        const int pos0 = lo0 + (int)threadIdx.x * step0, pos1 = lo1 + (int)threadIdx.x * step1;
        const int v0 = pos0 < hi0 ? a[pos0] : 0, v1 = pos1 < hi1 ? a[pos1] : 0;   // both loads before either count
        const int c0 = __syncthreads_count(pos0 < hi0 && v0 < g);
        const int c1 = __syncthreads_count(pos1 < hi1 && v1 < g + 1);
        if (lo0 < hi0) {
            if (c0 == 0) hi0 = lo0;
            else {
                const int nh = min(hi0, lo0 + c0 * step0);
                lo0 = lo0 + (c0 - 1) * step0 + 1;
                hi0 = nh;
            }
        }
        if (lo1 < hi1) {
            if (c1 == 0) hi1 = lo1;
            else {
                const int nh = min(hi1, lo1 + c1 * step1);
                lo1 = lo1 + (c1 - 1) * step1 + 1;
                hi1 = nh;
            }
        }
    }
    *first = lo0;
    *last = lo1;
}

template <bool MAX>
__global__ __launch_bounds__(kThreads) void pool_kernel(const int32_t *__restrict__ gi, int32_t N, const float *__restrict__ x,
                                                        int32_t F, int32_t lanes /* power of two <= 256 */, int mean,
                                                        float *__restrict__ out)
{
    __shared__ float part[kThreads];
    const int g = blockIdx.x;
    int lo, hi;
    block_run_bounds(gi, N, g, &lo, &hi);
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

// Few, large graphs (needs a workspace): `slices` blocks per graph.
//   FOLD == false: block (g, s) reduces the s-th of `slices` equal parts of graph g's run of rows of x into
//                  partial[g * slices + s][:]; block (g, 0) also writes the graph's node count to counts[g].
//   FOLD == true:  block g reduces the `slices` rows partial[g * slices ..][:] (read through x) and finishes as
//                  pool_kernel does: an empty graph gives 0, the mean divides by the node count.
// Threads are (row slot, column-group lane); a lane holds VEC neighbouring columns (VEC = 4: 128-bit loads, F % 4 == 0
// and 16-byte aligned rows); row slots stride over the rows and are combined through LDS in slot order, parts in
// part order: the result does not depend on scheduling.
template <bool MAX, int VEC, bool FOLD>
__global__ __launch_bounds__(kThreads) void pool_parts_kernel(const int32_t *__restrict__ gi, int32_t N,
                                                              const float *__restrict__ x, int32_t F,
                                                              int32_t lanes /* power of two <= 256 */, int mean,
                                                              int slices, int32_t *__restrict__ counts,
                                                              float *__restrict__ out)
{
    __shared__ float part[kThreads * VEC];
    int lo, hi;
    int64_t out_row;
    int cnt = 1;
    if constexpr (FOLD) {
        lo = (int)blockIdx.x * slices;
        hi = lo + slices;
        out_row = blockIdx.x;
        cnt = counts[blockIdx.x];
    } else {
        const int g = blockIdx.x / slices, slice = blockIdx.x % slices;
        block_run_bounds(gi, N, g, &lo, &hi);
        if (slice == 0 && threadIdx.x == 0) counts[g] = hi - lo;
        const int64_t len = hi - lo;
        const int first = lo + (int)(len * slice / slices), last = lo + (int)(len * (slice + 1) / slices);
        lo = first;
        hi = last;
        out_row = blockIdx.x;
    }
    const int fl = threadIdx.x % lanes, slot = threadIdx.x / lanes, slots = kThreads / lanes;
    const int fv = F / VEC;   // column groups
    for (int f0 = 0; f0 < fv; f0 += lanes) {
        const int f = f0 + fl;
        float acc[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc[c] = MAX ? -INFINITY : 0.0f;
        if (f < fv) {
#pragma unroll 4
            for (int i = lo + slot; i < hi; i += slots) {
                float v[VEC];
                if constexpr (VEC == 4) {
                    const float4 t = *reinterpret_cast<const float4 *>(x + (int64_t)i * F + f * 4);
                    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
                } else {
                    v[0] = x[(int64_t)i * F + f];
                }
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = MAX ? max_pz(acc[c], v[c]) : acc[c] + v[c];
            }
        }
#pragma unroll
        for (int c = 0; c < VEC; ++c) part[threadIdx.x * VEC + c] = acc[c];
        __syncthreads();
        if (slot == 0 && f < fv) {
            for (int s = 1; s < slots; ++s) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) {
                    const float v = part[(s * lanes + fl) * VEC + c];
                    acc[c] = MAX ? max_pz(acc[c], v) : acc[c] + v;
                }
            }
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                if constexpr (FOLD) {
                    if (cnt == 0) acc[c] = 0.0f;
                    if (mean && cnt > 0) acc[c] = acc[c] / (float)cnt;
                }
                out[out_row * F + f * VEC + c] = acc[c];
            }
        }
        __syncthreads();
    }
}

// The same search by one wavefront (64 probes per round, ballots instead of block-wide counts).
__device__ __forceinline__ void wave_run_bounds(const int32_t *__restrict__ gi, int N, int g, int lane, int *first,
                                                int *last)
{
    int lo0 = 0, hi0 = N, lo1 = 0, hi1 = N;
    while (lo0 < hi0 || lo1 < hi1) {   // wavefront-uniform
        const int step0 = max(1, (hi0 - lo0 + 63) / 64), step1 = max(1, (hi1 - lo1 + 63) / 64);
        const int pos0 = lo0 + lane * step0, pos1 = lo1 + lane * step1;
        const int v0 = pos0 < hi0 ? gi[pos0] : 0, v1 = pos1 < hi1 ? gi[pos1] : 0;
        const int c0 = __popcll(__ballot(pos0 < hi0 && v0 < g));
        const int c1 = __popcll(__ballot(pos1 < hi1 && v1 < g + 1));
        if (lo0 < hi0) {
            if (c0 == 0) hi0 = lo0;
            else {
                const int nh = min(hi0, lo0 + c0 * step0);
                lo0 = lo0 + (c0 - 1) * step0 + 1;
                hi0 = nh;
            }
        }
        if (lo1 < hi1) {
            if (c1 == 0) hi1 = lo1;
            else {
                const int nh = min(hi1, lo1 + c1 * step1);
                lo1 = lo1 + (c1 - 1) * step1 + 1;
                hi1 = nh;
            }
        }
    }
    *first = lo0;
    *last = lo1;
}

// Batches of small graphs: one wavefront per graph (four graphs per block), no block-wide barriers.  The run's
// bounds come from the same interleaved search with 64 probes per round; lanes are (node slot, feature lane),
// node slots stride over the run and are combined by a fixed xor-shuffle tree.
// VEC = 4: a feature lane holds four neighbouring columns (128-bit loads; F % 4 == 0, rows 16-byte aligned), which
// leaves four times as many node slots per wavefront.
template <bool MAX, int VEC>
__global__ __launch_bounds__(kThreads) void pool_wave_kernel(const int32_t *__restrict__ gi, int32_t N,
                                                             const float *__restrict__ x, int32_t F,
                                                             int32_t lanes /* power of two <= 64 */, int mean,
                                                             int32_t num_graphs, float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (g >= num_graphs) return;   // wavefront-uniform
    int lo, hi;
    wave_run_bounds(gi, N, g, lane, &lo, &hi);
    const int cnt = hi - lo;
    const int fl = lane % lanes, slot = lane / lanes, slots = 64 / lanes;
    const int fv = F / VEC;   // column groups
    for (int f0 = 0; f0 < fv; f0 += lanes) {
        const int f = f0 + fl;
        float acc[VEC];
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc[c] = MAX ? -INFINITY : 0.0f;
        if (f < fv) {
#pragma unroll 4
            for (int i = lo + slot; i < hi; i += slots) {
                float v[VEC];
                if constexpr (VEC == 4) {
                    const float4 t = *reinterpret_cast<const float4 *>(x + (int64_t)i * F + f * 4);
                    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
                } else {
                    v[0] = x[(int64_t)i * F + f];
                }
#pragma unroll
                for (int c = 0; c < VEC; ++c) acc[c] = MAX ? max_pz(acc[c], v[c]) : acc[c] + v[c];
            }
        }
        for (int off = lanes; off < 64; off <<= 1) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                const float other = __shfl_xor(acc[c], off, 64);
                acc[c] = MAX ? max_pz(acc[c], other) : acc[c] + other;
            }
        }
        if (slot == 0 && f < fv) {
#pragma unroll
            for (int c = 0; c < VEC; ++c) {
                if (cnt == 0) acc[c] = 0.0f;
                if (mean && cnt > 0) acc[c] = acc[c] / (float)cnt;
                out[(int64_t)g * F + f * VEC + c] = acc[c];
            }
        }
    }
}

// Backward of sum / mean pooling: every node of graph g receives gout[g,:] (divided by the node count for
// the mean).  One block per graph, same run search as the forward kernel; rows are written coalesced.
// relu_y (optional, [N x F]): the pooled rows were relu outputs; the gradient is zeroed where they are not positive
// (the relu's backward in the same pass).
__global__ __launch_bounds__(kThreads) void pool_backward_kernel(const int32_t *__restrict__ gi, int32_t N,
                                                                 const float *__restrict__ gout, int32_t F, int mean,
                                                                 const float *__restrict__ relu_y,
                                                                 float *__restrict__ gx)
{
    const int g = blockIdx.x;
    int lo, hi;
    block_run_bounds(gi, N, g, &lo, &hi);
    const int cnt = hi - lo;
    if (cnt <= 0) return;   // block-uniform
    const int64_t total = (int64_t)cnt * F;
    for (int64_t q = threadIdx.x; q < total; q += kThreads) {
        const int f = (int)(q % F);
        float v = gout[(int64_t)g * F + f];
        if (mean) v = v / (float)cnt;
        if (relu_y) v = relu_y[(int64_t)lo * F + q] > 0.0f ? v : 0.0f;
        gx[(int64_t)lo * F + q] = v;
    }
}

// The same for batches of many small graphs: one wavefront per graph.
__global__ __launch_bounds__(kThreads) void pool_backward_wave_kernel(const int32_t *__restrict__ gi, int32_t N,
                                                                      const float *__restrict__ gout, int32_t F,
                                                                      int mean, int32_t num_graphs,
                                                                      const float *__restrict__ relu_y,
                                                                      float *__restrict__ gx)
{
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.x * (kThreads / 64) + (threadIdx.x >> 6);
    if (g >= num_graphs) return;   // wavefront-uniform
    int lo, hi;
    wave_run_bounds(gi, N, g, lane, &lo, &hi);
    const int cnt = hi - lo;
    if (cnt <= 0) return;
    uintptr_t align = reinterpret_cast<uintptr_t>(gout) | reinterpret_cast<uintptr_t>(gx);
    if (relu_y) align |= reinterpret_cast<uintptr_t>(relu_y);
    if (F % 4 == 0 && (align & 15u) == 0) {
        const int fv = F / 4;
        const int64_t total = (int64_t)cnt * fv;
#pragma unroll 4
        for (int64_t q = lane; q < total; q += 64) {
            const int f = (int)(q % fv);
            float4 v = *reinterpret_cast<const float4 *>(gout + (int64_t)g * F + f * 4);
            if (mean) v = make_float4(v.x / (float)cnt, v.y / (float)cnt, v.z / (float)cnt, v.w / (float)cnt);
            if (relu_y) {
                const float4 y = *reinterpret_cast<const float4 *>(relu_y + (int64_t)lo * F + q * 4);
                v = make_float4(y.x > 0.0f ? v.x : 0.0f, y.y > 0.0f ? v.y : 0.0f, y.z > 0.0f ? v.z : 0.0f,
                                y.w > 0.0f ? v.w : 0.0f);
            }
            *reinterpret_cast<float4 *>(gx + (int64_t)lo * F + q * 4) = v;
        }
    } else {
        const int64_t total = (int64_t)cnt * F;
        for (int64_t q = lane; q < total; q += 64) {
            const int f = (int)(q % F);
            float v = gout[(int64_t)g * F + f];
            if (mean) v = v / (float)cnt;
            if (relu_y) v = relu_y[(int64_t)lo * F + q] > 0.0f ? v : 0.0f;
            gx[(int64_t)lo * F + q] = v;
        }
    }
}

// flags[0] |= 1 for a value outside [0, G), |= 2 for a descent between neighbours.
__global__ __launch_bounds__(kThreads) void check_indicator_kernel(const int32_t *__restrict__ gi, int32_t N, int32_t G,
                                                                   int32_t *__restrict__ flags)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    int bad = 0;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < N; i += stride) {
        const int32_t v = gi[i];
        if ((uint32_t)v >= (uint32_t)G) bad |= 1;
        if (i + 1 < N && gi[i + 1] < v) bad |= 2;
    }
    if (bad) atomicOr(flags, bad);
}

}  // namespace

extern "C" gnn_status gnn_check_graph_indicator(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                                void *stream)
{
    if (num_nodes < 0 || num_graphs <= 0) return GNN_ERR_BAD_SIZE;
    if (num_nodes == 0) return GNN_OK;
    if (!d_graph_indicator) return GNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    gnn_temp_pool pool;
    int32_t *d_flags = nullptr;
    GNN_TRY(pool.get(&d_flags, 1));
    GNN_HIP(hipMemsetAsync(d_flags, 0, sizeof(int32_t), s));
    const int blocks = (int)(gnn_div_up(num_nodes, kThreads) < 4096 ? gnn_div_up(num_nodes, kThreads) : 4096);
    hipLaunchKernelGGL(check_indicator_kernel, dim3(blocks), dim3(kThreads), 0, s, d_graph_indicator, num_nodes,
                       num_graphs, d_flags);
    GNN_LAUNCH_CHECK();
    int32_t h = 0;
    GNN_HIP(hipMemcpyAsync(&h, d_flags, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    GNN_HIP(hipStreamSynchronize(s));
    if (h & 1) return GNN_ERR_INDEX_RANGE;
    if (h & 2) return GNN_ERR_NOT_SORTED;
    return GNN_OK;
}

gnn_status gnn_launch_pool_backward(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                    const float *d_grad_out, int32_t feat_dim, gnn_aggr aggr, const float *d_relu_y,
                                    float *d_grad_x, hipStream_t stream)
{
    if (num_nodes < 0 || num_graphs <= 0 || feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (aggr == GNN_AGGR_MAX || aggr == GNN_AGGR_MIN || aggr == GNN_AGGR_PROD) return GNN_ERR_UNSUPPORTED;
    if (aggr != GNN_AGGR_SUM && aggr != GNN_AGGR_MEAN) return GNN_ERR_BAD_SIZE;
    if (num_nodes == 0) return GNN_OK;
    if (!d_graph_indicator || !d_grad_out || !d_grad_x) return GNN_ERR_NULL;
    const int mean = aggr == GNN_AGGR_MEAN ? 1 : 0;
    if ((int64_t)num_nodes <= (int64_t)num_graphs * kSmallGraphNodes && num_graphs >= kManyGraphs)
        hipLaunchKernelGGL(pool_backward_wave_kernel, dim3((unsigned)gnn_div_up(num_graphs, kThreads / 64)),
                           dim3(kThreads), 0, stream, d_graph_indicator, num_nodes, d_grad_out, feat_dim, mean,
                           num_graphs, d_relu_y, d_grad_x);
    else
        hipLaunchKernelGGL(pool_backward_kernel, dim3((unsigned)num_graphs), dim3(kThreads), 0, stream,
                           d_graph_indicator, num_nodes, d_grad_out, feat_dim, mean, d_relu_y, d_grad_x);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

extern "C" gnn_status gnn_graph_pool_backward(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                              const float *d_grad_out, int32_t feat_dim, gnn_aggr aggr,
                                              float *d_grad_x, void *stream)
{
    return gnn_launch_pool_backward(d_graph_indicator, num_nodes, num_graphs, d_grad_out, feat_dim, aggr, nullptr,
                                    d_grad_x, static_cast<hipStream_t>(stream));
}

namespace {

constexpr int kLargeGraphNodes = 8192;   // average nodes per graph from which a graph is worth several blocks
constexpr int kSliceNodes = 1024;        // ... of about this many nodes each,
constexpr int kMaxSlices = 1024;         // at most this many per graph

// Blocks per graph on the path with a workspace (1: the workspace is not used).
int pool_slices(int32_t num_nodes, int32_t num_graphs)
{
    if (num_graphs <= 0 || (int64_t)num_nodes < (int64_t)num_graphs * kLargeGraphNodes) return 1;
    const int64_t avg = num_nodes / num_graphs;
    return (int)std::min<int64_t>(kMaxSlices, gnn_div_up(avg, kSliceNodes));
}

size_t align256(size_t bytes) { return (bytes + 255) & ~(size_t)255; }

gnn_status pool_impl(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs, const float *d_x,
                     int32_t feat_dim, gnn_aggr aggr, float *d_out, void *d_workspace, size_t workspace_bytes,
                     void *stream);

}  // namespace

extern "C" size_t gnn_graph_pool_workspace_bytes(int32_t num_nodes, int32_t num_graphs, int32_t feat_dim)
{
    if (num_nodes <= 0 || num_graphs <= 0 || feat_dim <= 0) return 0;
    const int slices = pool_slices(num_nodes, num_graphs);
    if (slices <= 1) return 0;
    return align256((size_t)num_graphs * slices * feat_dim * sizeof(float)) + align256((size_t)num_graphs * sizeof(int32_t));
}

extern "C" gnn_status gnn_graph_pool(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                     const float *d_x, int32_t feat_dim, gnn_aggr aggr, float *d_out, void *stream)
{
    return pool_impl(d_graph_indicator, num_nodes, num_graphs, d_x, feat_dim, aggr, d_out, nullptr, 0, stream);
}

extern "C" gnn_status gnn_graph_pool_ws(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                        const float *d_x, int32_t feat_dim, gnn_aggr aggr, float *d_out,
                                        void *d_workspace, size_t workspace_bytes, void *stream)
{
    const size_t need = gnn_graph_pool_workspace_bytes(num_nodes, num_graphs, feat_dim);
    if (need > 0) {
        if (!d_workspace) return GNN_ERR_NULL;
        if (workspace_bytes < need || (reinterpret_cast<uintptr_t>(d_workspace) & 255u) != 0) return GNN_ERR_BAD_SIZE;
    }
    return pool_impl(d_graph_indicator, num_nodes, num_graphs, d_x, feat_dim, aggr, d_out, need ? d_workspace : nullptr,
                     need, stream);
}

namespace {

gnn_status pool_impl(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs, const float *d_x,
                     int32_t feat_dim, gnn_aggr aggr, float *d_out, void *d_workspace, size_t workspace_bytes,
                     void *stream)
{
    if (!d_out) return GNN_ERR_NULL;
    if (num_nodes < 0 || num_graphs <= 0 || feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (aggr != GNN_AGGR_SUM && aggr != GNN_AGGR_MEAN && aggr != GNN_AGGR_MAX) return GNN_ERR_BAD_SIZE;
    if (num_nodes > 0 && (!d_graph_indicator || !d_x)) return GNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int mean = aggr == GNN_AGGR_MEAN ? 1 : 0;
    // many small graphs: a wavefront each (with few graphs the block-per-graph kernel has more loads in flight)
    if ((int64_t)num_nodes <= (int64_t)num_graphs * kSmallGraphNodes && num_graphs >= kManyGraphs) {
        const bool vec4 = feat_dim % 4 == 0 && (reinterpret_cast<uintptr_t>(d_x) & 15u) == 0;
        const int groups = vec4 ? feat_dim / 4 : feat_dim;
        int lanes = 1;
        while (lanes < groups && lanes < 64) lanes <<= 1;
        const dim3 grid((unsigned)gnn_div_up(num_graphs, kThreads / 64));
        if (aggr == GNN_AGGR_MAX) {
            if (vec4)
                hipLaunchKernelGGL((pool_wave_kernel<true, 4>), grid, dim3(kThreads), 0, s, d_graph_indicator, num_nodes,
                                   d_x, feat_dim, lanes, 0, num_graphs, d_out);
            else
                hipLaunchKernelGGL((pool_wave_kernel<true, 1>), grid, dim3(kThreads), 0, s, d_graph_indicator, num_nodes,
                                   d_x, feat_dim, lanes, 0, num_graphs, d_out);
        } else {
            if (vec4)
                hipLaunchKernelGGL((pool_wave_kernel<false, 4>), grid, dim3(kThreads), 0, s, d_graph_indicator, num_nodes,
                                   d_x, feat_dim, lanes, mean, num_graphs, d_out);
            else
                hipLaunchKernelGGL((pool_wave_kernel<false, 1>), grid, dim3(kThreads), 0, s, d_graph_indicator, num_nodes,
                                   d_x, feat_dim, lanes, mean, num_graphs, d_out);
        }
        GNN_LAUNCH_CHECK();
        return GNN_OK;
    }
    // few large graphs and a workspace: several blocks per graph, parts combined in a fixed order afterwards
    const int slices = d_workspace ? pool_slices(num_nodes, num_graphs) : 1;
    if (slices > 1) {
        (void)workspace_bytes;   // checked by the caller against gnn_graph_pool_workspace_bytes
        float *partial = static_cast<float *>(d_workspace);
        int32_t *counts = reinterpret_cast<int32_t *>(static_cast<char *>(d_workspace) +
                                                      align256((size_t)num_graphs * slices * feat_dim * sizeof(float)));
        const bool vec4 = feat_dim % 4 == 0 && (reinterpret_cast<uintptr_t>(d_x) & 15u) == 0;   // stores are scalar
        const int groups = vec4 ? feat_dim / 4 : feat_dim;
        int lanes = 1;
        while (lanes < groups && lanes < kThreads) lanes <<= 1;
        const dim3 pgrid((unsigned)((int64_t)num_graphs * slices)), fgrid((unsigned)num_graphs);
#define GNN_POOL_PARTS(MAXV, VECV)                                                                                   \
    do {                                                                                                            \
        hipLaunchKernelGGL((pool_parts_kernel<MAXV, VECV, false>), pgrid, dim3(kThreads), 0, s, d_graph_indicator,  \
                           num_nodes, d_x, feat_dim, lanes, 0, slices, counts, partial);                            \
        GNN_LAUNCH_CHECK();                                                                                         \
        hipLaunchKernelGGL((pool_parts_kernel<MAXV, VECV, true>), fgrid, dim3(kThreads), 0, s,                      \
                           (const int32_t *)nullptr, 0, partial, feat_dim, lanes, mean, slices, counts, d_out);     \
        GNN_LAUNCH_CHECK();                                                                                         \
    } while (0)
        if (aggr == GNN_AGGR_MAX) {
            if (vec4) GNN_POOL_PARTS(true, 4);
            else GNN_POOL_PARTS(true, 1);
        } else {
            if (vec4) GNN_POOL_PARTS(false, 4);
            else GNN_POOL_PARTS(false, 1);
        }
#undef GNN_POOL_PARTS
        return GNN_OK;
    }
    int lanes = 1;
    while (lanes < feat_dim && lanes < kThreads) lanes <<= 1;
    if (aggr == GNN_AGGR_MAX)
        hipLaunchKernelGGL(pool_kernel<true>, dim3((unsigned)num_graphs), dim3(kThreads), 0, s, d_graph_indicator,
                           num_nodes, d_x, feat_dim, lanes, 0, d_out);
    else
        hipLaunchKernelGGL(pool_kernel<false>, dim3((unsigned)num_graphs), dim3(kThreads), 0, s, d_graph_indicator,
                           num_nodes, d_x, feat_dim, lanes, mean, d_out);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

}  // namespace
