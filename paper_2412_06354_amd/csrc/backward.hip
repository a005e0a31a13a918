// Backward of propagate: given g = dL/d out, the gradients with respect to the node features and
// the edge data.  The paper's purpose is training (its example differentiates through the layers,
// section 3 "Training Example"); the forward definition is that of section 3, "Message Passing".
//
//   sum : dL/dx[j,:] = sum_{k: src[k]=j} w[k,:] * g[dst[k],:]   -- a propagate over the graph sorted by
//         SOURCE (built by the caller with the roles of src and dst exchanged), gathering rows of g;
//         the edge data stay in the caller's edge order, which both graphs share through their perm.
//         dL/de[k] = <x[src[k],:], g[dst[k],:]>  (one weight per edge)  or the element-wise product:
//         one sub-group per edge of the by-destination CSR, perfectly balanced, two row gathers.
//   mean: the same with g[i,:] / in-degree(i) (scaled once into the workspace).
//   max : only the winning edge of every output element carries gradient.  The winners are found
//         by gnn_propagate_argmax from the forward result: per edge and feature the message is
//         recomputed and, where it is bit-identical to the maximum, the edge's CSR position enters an
//         integer atomic minimum (order-independent, hence deterministic), so ties go to the first
//         edge; positions are then translated to edge ids.  The backward kernels compare those ids.
#include "gnn_internal.h"

#include <algorithm>

namespace {

constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void scale_rows_by_inverse_degree_kernel(const int32_t *__restrict__ indeg,
                                                                               int64_t N, int F,
                                                                               const float *__restrict__ g,
                                                                               float *__restrict__ out)
{
    const int64_t total = N * F;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total; idx += stride) {
        const int d = indeg[idx / F];
        out[idx] = d > 0 ? g[idx] / (float)d : 0.0f;
    }
}

template <int VEC>
__device__ __forceinline__ void load_vec(float (&v)[VEC], const float *__restrict__ p)
{
    if constexpr (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = *p;
    }
}

// One sub-group of LPR lanes per CSR position q (edge perm[q] from colidx[q] to rowidx[q]); a lane owns
// VEC features per column block.  EVEC: element-wise edge data (no reduction), else one dot product.
// winners (or NULL): only features whose recorded winner is this edge contribute (max aggregation).
template <int LPR, int VEC, bool EVEC>
__global__ __launch_bounds__(kThreads) void edge_gradient_kernel(const int32_t *__restrict__ rowidx,
                                                                 const int32_t *__restrict__ colidx,
                                                                 const int32_t *__restrict__ perm, int64_t E, int F,
                                                                 const float *__restrict__ x,
                                                                 const float *__restrict__ gp,
                                                                 const int32_t *__restrict__ winners,
                                                                 float *__restrict__ grad_e)
{
    const int sl = threadIdx.x % LPR;
    const int64_t q = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / LPR;
    const bool have = q < E;   // no early return: the shuffles below run with every lane active
    const int64_t qc = have ? q : E - 1;
    const int64_t i = rowidx[qc], j = colidx[qc], k = perm[qc];
    float dot = 0.0f;
    for (int cb = 0; cb * LPR * VEC < F; ++cb) {
        const int col = (cb * LPR + sl) * VEC;
        if (col < F) {
            float xv[VEC], gv[VEC];
            load_vec<VEC>(xv, x + j * F + col);
            load_vec<VEC>(gv, gp + i * F + col);
            if (winners) {
                float wv[VEC];   // edge ids as raw bits
                load_vec<VEC>(wv, reinterpret_cast<const float *>(winners) + i * F + col);
#pragma unroll
                for (int c = 0; c < VEC; ++c)
                    if (__float_as_int(wv[c]) != (int)k) gv[c] = 0.0f;
            }
            if constexpr (EVEC) {
                if (have) {
#pragma unroll
                    for (int c = 0; c < VEC; ++c) grad_e[k * F + col + c] = xv[c] * gv[c];
                }
            } else {
#pragma unroll
                for (int c = 0; c < VEC; ++c) dot = fmaf(xv[c], gv[c], dot);
            }
        }
    }
    if constexpr (!EVEC) {
#pragma unroll
        for (int off = LPR / 2; off > 0; off >>= 1) dot += __shfl_xor(dot, off, LPR);
        if (have && sl == 0) grad_e[k] = dot;
    }
}

template <int LPR, int VEC>
gnn_status launch_edge_gradient(const gnn_graph *g, int F, bool evec, const float *x, const float *gp,
                                const int32_t *winners, float *grad_e, hipStream_t s)
{
    const int64_t blocks = gnn_div_up(g->num_edges * LPR, kThreads);
    if (evec)
        hipLaunchKernelGGL((edge_gradient_kernel<LPR, VEC, true>), dim3((unsigned)blocks), dim3(kThreads), 0, s,
                           g->rowidx, g->colidx, g->perm, g->num_edges, F, x, gp, winners, grad_e);
    else
        hipLaunchKernelGGL((edge_gradient_kernel<LPR, VEC, false>), dim3((unsigned)blocks), dim3(kThreads), 0, s,
                           g->rowidx, g->colidx, g->perm, g->num_edges, F, x, gp, winners, grad_e);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

// ---------------------------------------------------------------- winners of a max aggregation

__global__ __launch_bounds__(kThreads) void fill_i32_kernel(int32_t *__restrict__ a, int64_t n, int32_t v)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) a[i] = v;
}

// Thread per (CSR position q, feature): recompute the message; where it is bit-identical to the row's
// maximum, q enters the element's atomic minimum.  E_KIND: 0 copy_xj, 1 one weight per edge, 2 element-wise.
template <int E_KIND>
__global__ __launch_bounds__(kThreads) void match_max_kernel(const int32_t *__restrict__ rowidx,
                                                             const int32_t *__restrict__ colidx,
                                                             const int32_t *__restrict__ perm, int64_t E, int F,
                                                             const float *__restrict__ x, const float *__restrict__ e,
                                                             int e_coo, const float *__restrict__ out_max,
                                                             int32_t *__restrict__ first_pos)
{
    const int64_t total = E * F;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total; idx += stride) {
        const int64_t q = idx / F;
        const int f = (int)(idx - q * F);
        const int64_t i = rowidx[q], j = colidx[q];
        float m = x[j * F + f];
        if constexpr (E_KIND != 0) {
            const int64_t eid = e_coo ? perm[q] : q;
            m = (E_KIND == 1 ? e[eid] : e[eid * F + f]) * m;
        }
        if (__float_as_int(m) == __float_as_int(out_max[i * F + f])) atomicMin(first_pos + i * F + f, (int32_t)q);
    }
}

__global__ __launch_bounds__(kThreads) void positions_to_edge_ids_kernel(const int32_t *__restrict__ perm, int64_t n,
                                                                        int32_t *__restrict__ a)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const int32_t q = a[i];
        a[i] = q == INT32_MAX ? -1 : perm[q];
    }
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" {

size_t gnn_propagate_backward_workspace_bytes(int32_t num_nodes, int32_t feat_dim, gnn_aggr aggr)
{
    if (num_nodes <= 0 || feat_dim <= 0 || aggr != GNN_AGGR_MEAN) return 0;
    return (size_t)num_nodes * feat_dim * sizeof(float);
}

gnn_status gnn_propagate_argmax(const gnn_graph *g, const float *d_x, int32_t feat_dim, const float *d_e,
                                int32_t e_dim, gnn_edge_order e_order, gnn_msg_op msg, const float *d_out_max,
                                int32_t *d_argmax, void *stream)
{
    if (!g || !d_argmax) return GNN_ERR_NULL;
    if (feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (msg != GNN_MSG_COPY_XJ && msg != GNN_MSG_E_MUL_XJ) return GNN_ERR_BAD_SIZE;
    if (msg == GNN_MSG_E_MUL_XJ) {
        if (e_dim != 1 && e_dim != feat_dim) return GNN_ERR_BAD_SIZE;
        if (e_order != GNN_EDGE_ORDER_COO && e_order != GNN_EDGE_ORDER_CSR) return GNN_ERR_BAD_SIZE;
        if (!d_e && g->num_edges > 0) return GNN_ERR_NULL;
    }
    if (g->num_edges > 0 && (!d_x || !d_out_max)) return GNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int F = feat_dim;
    const int64_t nf = (int64_t)g->num_nodes * F;
    const int fill_blocks = (int)std::min<int64_t>(gnn_div_up(nf, kThreads), 256 * 64);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(fill_blocks), dim3(kThreads), 0, s, d_argmax, nf, INT32_MAX);
    GNN_LAUNCH_CHECK();
    if (g->num_edges > 0) {
        const int blocks = (int)std::min<int64_t>(gnn_div_up(g->num_edges * F, kThreads), 256 * 256);
        const int e_coo = (e_order == GNN_EDGE_ORDER_COO);
        const int kind = msg == GNN_MSG_COPY_XJ ? 0 : (e_dim == 1 ? 1 : 2);
        if (kind == 0)
            hipLaunchKernelGGL(match_max_kernel<0>, dim3(blocks), dim3(kThreads), 0, s, g->rowidx, g->colidx, g->perm,
                               g->num_edges, F, d_x, d_e, e_coo, d_out_max, d_argmax);
        else if (kind == 1)
            hipLaunchKernelGGL(match_max_kernel<1>, dim3(blocks), dim3(kThreads), 0, s, g->rowidx, g->colidx, g->perm,
                               g->num_edges, F, d_x, d_e, e_coo, d_out_max, d_argmax);
        else
            hipLaunchKernelGGL(match_max_kernel<2>, dim3(blocks), dim3(kThreads), 0, s, g->rowidx, g->colidx, g->perm,
                               g->num_edges, F, d_x, d_e, e_coo, d_out_max, d_argmax);
        GNN_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(positions_to_edge_ids_kernel, dim3(fill_blocks), dim3(kThreads), 0, s, g->perm, nf, d_argmax);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_propagate_backward(const gnn_graph *g, const gnn_graph *g_by_source, const float *d_x,
                                  int32_t feat_dim, const float *d_e, int32_t e_dim, gnn_msg_op msg, gnn_aggr aggr,
                                  const float *d_grad_out, const int32_t *d_argmax, float *d_grad_x,
                                  float *d_grad_e, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!g || !d_grad_out) return GNN_ERR_NULL;
    if (feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (msg != GNN_MSG_COPY_XJ && msg != GNN_MSG_E_MUL_XJ) return GNN_ERR_BAD_SIZE;
    if (aggr != GNN_AGGR_SUM && aggr != GNN_AGGR_MEAN && aggr != GNN_AGGR_MAX) return GNN_ERR_BAD_SIZE;
    if (aggr == GNN_AGGR_MAX && !d_argmax) return GNN_ERR_NULL;
    const int32_t *winners = aggr == GNN_AGGR_MAX ? d_argmax : nullptr;
    if (msg == GNN_MSG_E_MUL_XJ) {
        if (e_dim != 1 && e_dim != feat_dim) return GNN_ERR_BAD_SIZE;
        if (!d_e && g->num_edges > 0) return GNN_ERR_NULL;
    }
    if (d_grad_x) {
        if (!g_by_source) return GNN_ERR_NULL;
        if (g_by_source->num_nodes != g->num_nodes || g_by_source->num_edges != g->num_edges) return GNN_ERR_BAD_SIZE;
    }
    if (d_grad_e && msg == GNN_MSG_E_MUL_XJ && !d_x) return GNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int F = feat_dim;
    const int64_t N = g->num_nodes;

    const float *gp = d_grad_out;
    if (aggr == GNN_AGGR_MEAN) {
        if (!d_workspace) return GNN_ERR_NULL;
        if (workspace_bytes < gnn_propagate_backward_workspace_bytes(g->num_nodes, F, aggr)) return GNN_ERR_BAD_SIZE;
        if (!aligned16(d_workspace)) return GNN_ERR_BAD_SIZE;
        float *scaled = static_cast<float *>(d_workspace);
        const int blocks = (int)std::min<int64_t>(gnn_div_up(N * F, kThreads), 256 * 64);
        hipLaunchKernelGGL(scale_rows_by_inverse_degree_kernel, dim3(blocks), dim3(kThreads), 0, s, g->indeg, N, F,
                           d_grad_out, scaled);
        GNN_LAUNCH_CHECK();
        gp = scaled;
    }
    if (d_grad_x) {
        gnn_epilogue epi;
        GNN_TRY(gnn_launch_propagate(g_by_source, gp, F, d_e, e_dim, GNN_EDGE_ORDER_COO, msg, 0, epi, d_grad_x, s,
                                     GNN_GATHER_SOURCE_NODE, winners));
    }
    if (d_grad_e && msg == GNN_MSG_E_MUL_XJ && g->num_edges > 0) {
        const bool evec = (e_dim != 1);
        const bool vec4 = (F % 4 == 0) && aligned16(d_x) && aligned16(gp) && (!evec || aligned16(d_grad_e)) &&
                          aligned16(winners);
        if (vec4) {
            const int cols = F / 4;
            if (cols <= 4) return launch_edge_gradient<4, 4>(g, F, evec, d_x, gp, winners, d_grad_e, s);
            if (cols <= 8) return launch_edge_gradient<8, 4>(g, F, evec, d_x, gp, winners, d_grad_e, s);
            if (cols <= 16) return launch_edge_gradient<16, 4>(g, F, evec, d_x, gp, winners, d_grad_e, s);
            return launch_edge_gradient<32, 4>(g, F, evec, d_x, gp, winners, d_grad_e, s);
        }
        if (F <= 16) return launch_edge_gradient<16, 1>(g, F, evec, d_x, gp, winners, d_grad_e, s);
        return launch_edge_gradient<64, 1>(g, F, evec, d_x, gp, winners, d_grad_e, s);
    }
    return GNN_OK;
}

}  // extern "C"
