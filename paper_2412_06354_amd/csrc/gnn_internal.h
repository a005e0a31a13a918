// Internal declarations shared by the translation units of the library (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <vector>

#include "gnn.h"

// Turns a failing HIP call into GNN_ERR_DEVICE (or GNN_ERR_ALLOC for allocations).
#define GNN_HIP(call)                                  \
    do {                                               \
        hipError_t e_ = (call);                        \
        if (e_ != hipSuccess) {                        \
            (void)hipGetLastError();                   \
            return GNN_ERR_DEVICE;                     \
        }                                              \
    } while (0)

#define GNN_TRY(call)                  \
    do {                               \
        gnn_status s_ = (call);        \
        if (s_ != GNN_OK) return s_;   \
    } while (0)

#define GNN_LAUNCH_CHECK() GNN_HIP(hipGetLastError())

static inline int64_t gnn_div_up(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Device allocations that are released together (temporaries of one call).
struct gnn_temp_pool {
    std::vector<void *> ptrs;
    ~gnn_temp_pool() { release(); }
    void release() {
        for (void *p : ptrs) (void)hipFree(p);
        ptrs.clear();
    }
    template <typename T>
    gnn_status get(T **out, size_t count) {
        void *p = nullptr;
        if (hipMalloc(&p, (count ? count : 1) * sizeof(T)) != hipSuccess) {
            (void)hipGetLastError();
            return GNN_ERR_ALLOC;
        }
        ptrs.push_back(p);
        *out = static_cast<T *>(p);
        return GNN_OK;
    }
};

// One device allocation shared by the graphs of a batch build; freed when the last of them is destroyed.
struct shared_slab {
    void *ptr = nullptr;
    size_t bytes = 0;
    int device = -1;
    std::atomic<int> refs{0};
};

// Index arrays and buffers of the two-pass route that moves one float per edge between the caller's edge order and
// CSR order in streams (route.hip); built on request by gnn_graph_build_edge_route, one allocation.
struct gnn_edge_route {
    void *alloc = nullptr;
    uint16_t *tile_src = nullptr;     // [E] per tile of edge ids: local edge of the k-th item in (bucket, edge id) order
    int32_t *tile_dst = nullptr;      // [E] its place in `mid`
    uint16_t *bucket_idx = nullptr;   // [E] per bucket of CSR positions: where in the bucket of `mid` position p's value lies
    float *mid = nullptr;             // [E] the intermediate order, grouped by bucket
    float *staged = nullptr;          // [E] CSR-ordered copy of edge data for compute calls that are handed COO order
};

struct gnn_graph {
    int32_t num_nodes = 0;        // rows of the CSR = destination nodes
    int32_t num_src_nodes = 0;    // range of colidx; equals num_nodes unless built from a relation between two node sets
    bool bipartite = false;       // built by gnn_build_csr_bipartite: sources and destinations are different node sets
    int64_t num_edges = 0;
    int32_t small_max = 0;   // rows with in-degree <= small_max: one sub-group of a wavefront each
    int32_t chunk = 0;       // longer rows: pieces of <= chunk edges, one wavefront each

    shared_slab *shared = nullptr;   // set when the arrays lie in a batch's allocation (slab is then unused)
    void *slab = nullptr;        // the one allocation holding every array below
    size_t slab_bytes = 0;       // its size, and the device it lives on (it may be handed to a later build)
    int device = -1;

    int32_t *rowptr = nullptr;   // [N+1]
    int32_t *indeg = nullptr;    // [N]
    int32_t *colidx = nullptr;   // [E]
    int32_t *perm = nullptr;     // [E]
    int32_t *rowidx = nullptr;   // [E] destination of CSR position p (the sorted keys)
    int32_t *dst_coo = nullptr;  // [E] destination of edge k in the caller's order (a copy of the input)
    float *dinv_loop = nullptr;  // [N] 1/sqrt(in-degree + 1): GCN coefficient with one self-loop per node
    float *dinv_plain = nullptr; // [N] 1/sqrt(in-degree), 0 where the in-degree is 0

    int32_t n_small = 0;
    int32_t *small_rows = nullptr;      // [n_small] row ids, ascending
    int32_t n_items = 0;
    int32_t *item_row = nullptr;        // [n_items]
    int32_t *item_start = nullptr;      // [n_items] first CSR position of the piece
    int32_t *item_slot = nullptr;       // [n_items] partial-result slot, or -1 if the piece is a whole row
    int32_t n_slots = 0;
    int32_t n_split = 0;
    int32_t *split_rows = nullptr;      // [n_split] rows made of several pieces
    int32_t *split_slot0 = nullptr;     // [n_split] first slot of the row (slots are consecutive)

    // Partial results of split rows and per-row statistics, shared by all compute calls on this graph.  Sized when
    // the graph is built (a part of the slab) and only ever replaced by gnn_graph_reserve: compute calls never
    // allocate, they fail with GNN_ERR_NOT_RESERVED when it is too small.
    float *scratch = nullptr;
    size_t scratch_floats = 0;
    void *own_scratch = nullptr;   // the allocation gnn_graph_reserve made, if any (scratch points into it)

    gnn_edge_route *route = nullptr;   // set by gnn_graph_build_edge_route
};

// out = in moved from the caller's edge order to CSR order / back, one float per edge, through the graph's route
// (GNN_ERR_UNSUPPORTED without one).  in and out are 16-byte aligned; the route's `mid` buffer is overwritten.
gnn_status gnn_route_coo_to_csr(const gnn_graph *g, const float *d_in, float *d_out, hipStream_t s);
gnn_status gnn_route_csr_to_coo(const gnn_graph *g, const float *d_in, float *d_out, hipStream_t s);
void gnn_route_free(gnn_graph *g);
static inline bool gnn_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Feature width the scratch part of the slab is sized for (see gnn_graph_reserve in gnn.h).
constexpr int32_t kDefaultReservedFeatDim = 128;

// Floats of scratch the compute calls need: three partial rows per slot for the widest user (the attention
// layer keeps a weighted sum, a maximum and a denominator per slot and feature), a (max, denominator) pair per
// row and slot and head for the segment softmax.
static inline size_t gnn_scratch_floats(int64_t slots, int32_t num_nodes, int32_t feat_dim, int32_t heads)
{
    const size_t a = 3 * (size_t)slots * (size_t)(feat_dim > 0 ? feat_dim : 0);
    const size_t b = 2 * ((size_t)num_nodes + (size_t)slots) * (size_t)(heads > 0 ? heads : 0);
    return a > b ? a : b;
}

// The graph's scratch buffer if it holds at least `floats` floats, else GNN_ERR_NOT_RESERVED.  Never allocates.
static inline gnn_status gnn_graph_scratch(const gnn_graph *g, size_t floats, float **out)
{
    *out = g->scratch;
    if (floats > g->scratch_floats) return GNN_ERR_NOT_RESERVED;
    return GNN_OK;
}

// sum_partials with a final factor: out[q] = factor * sum over chunks of partial[chunk * elems + q]
gnn_status gnn_launch_sum_partials_scaled(const float *d_partial, int chunks, int64_t elems, float factor,
                                          float *d_out, hipStream_t stream);

// Exclusive prefix sums along every row of a row-major [rows x cols] array, in place; d_row_totals[r] receives the
// sum of row r.
gnn_status gnn_scan_rows_exclusive_i32(int32_t *d_data, int rows, int64_t cols, int32_t *d_row_totals,
                                       hipStream_t stream);

// The same for several arrays with the same number of rows in one launch; d_jobs is a device array of num_jobs
// entries (cols may differ from job to job; a job with cols == 0 only gets zero totals).
struct gnn_scan_job {
    int32_t *data;
    int64_t cols;
    int32_t *row_totals;
};
gnn_status gnn_scan_rows_exclusive_i32_jobs(const gnn_scan_job *d_jobs, int num_jobs, int rows, hipStream_t stream);

// Epilogue applied to a finished row reduction:  out = act(post * (acc + self_scale * x[row]) + bias)
// with post = row_scale[row] (or 1), or acc / in-degree for the mean.
struct gnn_epilogue {
    int mean = 0;                    // divide by the in-degree (0 stays 0)
    float self_scale = 0.f;          // adds self_scale * x[row,:] when non-zero
    const float *row_scale = nullptr;
    const float *bias = nullptr;
    int relu = 0;                    // max(., 0) last
    int accumulate = 0;              // out += result instead of out = result (sum over relations)
    // copy_xj with sum only: edge j -> i carries source_scale[j] * x[j,:] and the self term becomes
    // self_scale * source_scale[row] * x[row,:]  (a diagonal scaling of x that is never written out)
    const float *source_scale = nullptr;
};

// Which row of `x` CSR position p gathers: x[colidx[p]] for node features (the default),
// x[perm[p]] for per-edge rows stored in the caller's edge order, x[p] for per-edge rows stored in
// CSR order.
enum gnn_gather_index { GNN_GATHER_SOURCE_NODE = 0, GNN_GATHER_EDGE_COO = 1, GNN_GATHER_EDGE_CSR = 2 };

// How a row's messages are reduced (the mean is a sum with gnn_epilogue::mean set).
enum gnn_reduce { GNN_REDUCE_SUM = 0, GNN_REDUCE_MAX = 1, GNN_REDUCE_MIN = 2, GNN_REDUCE_PROD = 3 };

// d_winners (optional, sum only, edge data in the caller's order): [rows of x][feat_dim] edge ids; a
// gathered element x[j,f] only contributes to the edge whose id equals d_winners[j,f] (the routing
// step of a max aggregation's backward pass).
// x_is_bf16: d_x points to bfloat16 values (copy_xj or one weight per edge, sum / mean / max, feat_dim % 8 == 0).
// d_scratch (optional): device buffer of scratch_floats floats that receives the partial rows of split rows instead
// of the graph's own scratch memory (GNN_ERR_SCRATCH_LIMIT if it is too small).
// Shared launcher behind gnn_propagate / gnn_aggregate_neighbors / gnn_gin_update / the sparse half
// of gnn_gcnconv.
gnn_status gnn_launch_propagate(const gnn_graph *g, const float *d_x, int32_t feat_dim,
                                const float *d_e, int32_t e_dim, gnn_edge_order e_order,
                                gnn_msg_op msg, int reduce, const gnn_epilogue &epi,
                                float *d_out, hipStream_t stream,
                                gnn_gather_index gather = GNN_GATHER_SOURCE_NODE,
                                const int32_t *d_winners = nullptr, int x_is_bf16 = 0,
                                float *d_scratch = nullptr, size_t scratch_floats = 0);

// out[k] = <x[src[k],:], y[dst[k],:]> per edge, in the order out_order names (backward.hip)
gnn_status gnn_launch_edge_dot(const gnn_graph *g, const float *d_x_src, const float *d_y_dst, int32_t feat_dim,
                               float *d_out, gnn_edge_order out_order, void *stream);

// ---- dense helpers shared by the backward passes (gcn_backward.hip)
// Number of row chunks the two-stage reductions over N rows use.
int gnn_row_chunk_count(int64_t rows);
// out[f_in x f_out] = X^T Y over `rows` rows (fp32 MFMA, fixed summation order).  d_partial holds
// gnn_row_chunk_count(rows) * f_in * f_out floats.
gnn_status gnn_launch_xty(const float *d_x, const float *d_y, int64_t rows, int f_in, int f_out, float *d_partial,
                          float *d_out, hipStream_t stream);
// out[q] = sum over chunks (fixed order) of partial[chunk * elems + q]
gnn_status gnn_launch_sum_partials(const float *d_partial, int chunks, int64_t elems, float *d_out,
                                   hipStream_t stream);
// Backward of sum / mean pooling; d_relu_y (optional, [N x F]) = the pooled rows when they were relu outputs: the
// relu's backward rides in the same pass (pool.hip).
gnn_status gnn_launch_pool_backward(const int32_t *d_graph_indicator, int32_t num_nodes, int32_t num_graphs,
                                    const float *d_grad_out, int32_t feat_dim, gnn_aggr aggr, const float *d_relu_y,
                                    float *d_grad_x, hipStream_t stream);
// A batch normalisation (with its optional relu) applied to the rows of X as they are read, so that the
// normalised matrix is never written:  x'[r,f] = act(gamma[f] * ((x[r,f] - mean[f]) / sqrt(var[f] + eps)) + beta[f]),
// the arithmetic of gnn_batchnorm's own pass, operation for operation.  gamma / beta may be null (1 / 0).
struct gnn_column_norm {
    const float *mean = nullptr, *var = nullptr, *gamma = nullptr, *beta = nullptr;
    float eps = 0.0f;
    int relu = 0;
};
// True if gnn_launch_xw would take the kernel that can apply a gnn_column_norm to X for this shape.
bool gnn_xw_takes_column_norm(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n);
// Z = X W with the store's epilogue: optional per-row scale, then per-column bias, then relu (gemm.hip).
// norm (optional): X is normalised on the way in; only where gnn_xw_takes_column_norm says so (else GNN_ERR_UNSUPPORTED).
gnn_status gnn_launch_xw(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                         const float *d_row_scale, const float *d_bias, bool relu, float *d_z, hipStream_t s,
                         const gnn_column_norm *norm = nullptr, bool w_transposed = false);
// w_transposed: d_w is stored [n x k] and the product is X d_w^T (the backward passes multiply by the transpose of
// the forward's weights); only where gnn_xw_takes_transposed_w says so (else GNN_ERR_UNSUPPORTED).
bool gnn_xw_takes_transposed_w(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n);
// Z = X W^T for W stored [n x k]: directly where the projection kernel can read W that way, else through a
// transposed copy in d_wt (n * k floats).
gnn_status gnn_launch_xwt(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                          const float *d_row_scale, float *d_wt, float *d_z, hipStream_t s);
// gnn_gcnconv with an optional batch normalisation of X applied as the projection reads it (gcnconv.hip); with a
// norm only where gnn_gcnconv_takes_column_norm says so.
bool gnn_gcnconv_takes_column_norm(const gnn_graph *g, const float *d_x, int32_t f_in, const float *d_w, int32_t f_out);
gnn_status gnn_launch_gcnconv(const gnn_graph *g, const float *d_x, int32_t f_in, const float *d_w, const float *d_bias,
                              int32_t f_out, int32_t add_self_loops, gnn_activation act, float *d_out,
                              void *d_workspace, size_t workspace_bytes, void *stream, const gnn_column_norm *norm);
// wt[cols x rows] = w[rows x cols]^T
gnn_status gnn_launch_transpose(const float *d_w, int rows, int cols, float *d_wt, hipStream_t stream);
// sl[i,hd] = <a_src[hd,:], h[i,hd,:]>, sr[i,hd] = <a_dst[hd,:], h[i,hd,:]>  (gatconv.hip)
gnn_status gnn_launch_node_scores(const float *d_h, int64_t N, int heads, int ch, const float *d_a_src,
                                  const float *d_a_dst, float *d_sl, float *d_sr, hipStream_t stream);

