// GCNConv forward,  out = D^-1/2 (A [+ I]) D^-1/2 X W + b  (layer used in the paper's training
// example; a fused special case of propagate in the sense of section 3, "Message Passing").
//
// Steps on the caller's stream:
//   1. dinv[i] = 1/sqrt(d_i),  d_i = in-degree (+1 with self-loops), 0 where d_i = 0 -- kept with the graph;
//   2. Z'[j,:] = dinv[j] * (X W)[j,:]      -- MFMA projection with the source-side factor fused in;
//   3. out[i,:] = dinv[i] * (sum_{j->i} Z'[j,:] + [self-loop] Z'[i,:]) + b   -- the propagate kernel
//      (copy_xj, sum) with the self-loop term, the destination-side factor and the bias applied in
//      its epilogue, so the self-loops are never materialised as edges; an optional relu (the
//      example model's second graph convolution, which has a relu) is applied there too.
// A layer that widens (f_in < f_out, the example model's first graph convolution, 16 to 64 features) runs in the other order, so that the gather
// moves rows of f_in values instead of f_out:
//   2'. T[i,:] = dinv[i] * (sum_{j->i} dinv[j] X[j,:] + [self-loop] dinv[i] X[i,:])   -- the propagate kernel with one
//       weight per edge looked up by source node (X is never rescaled in memory);
//   3'. out = T W + b  -- MFMA projection with bias and relu in its store.
#include "gnn_internal.h"

namespace {

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

}  // namespace

bool gnn_gcnconv_takes_column_norm(const gnn_graph *g, const float *d_x, int32_t f_in, const float *d_w, int32_t f_out)
{
    // the projection has to come first (it is what reads X), in the kernel that can normalise on the way in
    return g && f_in >= f_out && gnn_xw_takes_column_norm(d_x, g->num_nodes, f_in, d_w, f_out);
}

gnn_status gnn_launch_gcnconv(const gnn_graph *g, const float *d_x, int32_t f_in, const float *d_w, const float *d_bias,
                              int32_t f_out, int32_t add_self_loops, gnn_activation act, float *d_out,
                              void *d_workspace, size_t workspace_bytes, void *stream, const gnn_column_norm *norm)
{
    if (!g || !d_x || !d_w || !d_out || !d_workspace) return GNN_ERR_NULL;
    if (f_in <= 0 || f_out <= 0) return GNN_ERR_BAD_SIZE;
    if (act != GNN_ACT_NONE && act != GNN_ACT_RELU) return GNN_ERR_BAD_SIZE;
    if (g->bipartite) return GNN_ERR_UNSUPPORTED;   // one node set only: X has a row per node of the graph
    const int32_t N = g->num_nodes;
    if (workspace_bytes < gnn_gcnconv_workspace_bytes(N, f_out)) return GNN_ERR_BAD_SIZE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255u) return GNN_ERR_BAD_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float *z = static_cast<float *>(d_workspace);
    const float *dinv = add_self_loops ? g->dinv_loop : g->dinv_plain;   // computed when the graph was built

    if (f_in < f_out) {   // aggregate the narrow rows first
        gnn_epilogue agg;
        agg.self_scale = add_self_loops ? 1.0f : 0.0f;
        agg.row_scale = dinv;
        agg.source_scale = dinv;
        if (norm) return GNN_ERR_UNSUPPORTED;   // the gather reads X here
        GNN_TRY(gnn_launch_propagate(g, d_x, f_in, nullptr, 1, GNN_EDGE_ORDER_CSR, GNN_MSG_COPY_XJ, 0, agg, z, s));
        return gnn_launch_xw(z, N, f_in, d_w, f_out, nullptr, d_bias, act == GNN_ACT_RELU, d_out, s);
    }
    GNN_TRY(gnn_launch_xw(d_x, N, f_in, d_w, f_out, dinv, nullptr, false, z, s, norm));
    gnn_epilogue epi;
    epi.self_scale = add_self_loops ? 1.0f : 0.0f;
    epi.row_scale = dinv;
    epi.bias = d_bias;
    epi.relu = (act == GNN_ACT_RELU);
    return gnn_launch_propagate(g, z, f_out, nullptr, 1, GNN_EDGE_ORDER_CSR, GNN_MSG_COPY_XJ, 0, epi, d_out, s);
}

extern "C" {

size_t gnn_gcnconv_workspace_bytes(int32_t num_nodes, int32_t f_out)
{
    if (num_nodes <= 0 || f_out <= 0) return 0;
    return align256((size_t)num_nodes * f_out * sizeof(float));
}

gnn_status gnn_gcnconv(const gnn_graph *g, const float *d_x, int32_t f_in, const float *d_w, const float *d_bias,
                       int32_t f_out, int32_t add_self_loops, gnn_activation act, float *d_out,
                       void *d_workspace, size_t workspace_bytes, void *stream)
{
    return gnn_launch_gcnconv(g, d_x, f_in, d_w, d_bias, f_out, add_self_loops, act, d_out, d_workspace,
                              workspace_bytes, stream, nullptr);
}

}  // extern "C"
