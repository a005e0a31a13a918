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

// A wavefront takes 64 consecutive CSR positions (edge perm[q] from colidx[q] to rowidx[q]) per round: every
// lane fetches the indices of one position (coalesced), then each sub-group of LPR lanes walks over its own
// LPR consecutive positions in batches of U, a lane owning VEC features per column block; the row gathers of
// a batch are issued before their products are taken.  EVEC: element-wise edge data (rows written directly);
// else one dot product per position: the U partial dots a lane holds are folded by a halving exchange (a
// lane gives away the half it does not keep; U-1 shuffles for U positions) and then across the remaining
// lane bits, in a fixed order; lane t of the sub-group ends up with the total of its own position.
// WIN: only features whose recorded winner is this edge contribute (max aggregation); a template
// parameter because a run-time branch between the gathers would make the compiler wait for each of them.
template <int LPR, int VEC, bool EVEC, bool WIN>
__global__ __launch_bounds__(kThreads) void edge_gradient_kernel(const int32_t *__restrict__ rowidx,
                                                                 const int32_t *__restrict__ colidx,
                                                                 const int32_t *__restrict__ perm, int64_t E, int F,
                                                                 const float *__restrict__ x,
                                                                 const float *__restrict__ gp,
                                                                 const int32_t *__restrict__ winners,
                                                                 float *__restrict__ grad_e)
{
    constexpr int U = LPR < 8 ? LPR : 8;
    const int lane = threadIdx.x & 63, sl = lane % LPR;
    const int64_t waves = (int64_t)gridDim.x * (kThreads / 64);
    for (int64_t q0 = (((int64_t)blockIdx.x * kThreads + threadIdx.x) >> 6) * 64; q0 < E; q0 += waves * 64) {
        const int64_t q = q0 + lane;
        const bool have = q < E;
        const int64_t qc = have ? q : E - 1;   // clamped: loads stay in bounds, results are dropped
        const int i_own = rowidx[qc], j_own = colidx[qc], k_own = perm ? perm[qc] : (int)qc;   // no perm: CSR-ordered output
        const int64_t group_q0 = q0 + (lane - sl);
        float mine = 0.0f;
        for (int cb = 0; cb * LPR * VEC < F; ++cb) {
            const int col = (cb * LPR + sl) * VEC;
            const bool ok = col < F;
            const int colc = ok ? col : 0;
            for (int t0 = 0; t0 < LPR; t0 += U) {
                float xv[U][VEC], gv[U][VEC], d[U];
                int kk[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int64_t i = __shfl(i_own, t0 + u, LPR), j = __shfl(j_own, t0 + u, LPR);
                    load_vec<VEC>(xv[u], x + j * F + colc);
                    load_vec<VEC>(gv[u], gp + i * F + colc);
                    if constexpr (EVEC || WIN) kk[u] = __shfl(k_own, t0 + u, LPR);
                    if constexpr (WIN) {
                        float wv[VEC];   // edge ids as raw bits
                        load_vec<VEC>(wv, reinterpret_cast<const float *>(winners) + i * F + colc);
#pragma unroll
                        for (int c = 0; c < VEC; ++c)
                            if (__float_as_int(wv[c]) != kk[u]) gv[u][c] = 0.0f;
                    }
                }
                // all gathers of the batch are in flight before the first product: without the barrier the
                // scheduler interleaves them pairwise with the arithmetic to save registers
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (EVEC) {
                        if (ok && group_q0 + t0 + u < E) {
#pragma unroll
                            for (int c = 0; c < VEC; ++c) grad_e[(int64_t)kk[u] * F + col + c] = xv[u][c] * gv[u][c];
                        }
                    } else {
                        float acc = 0.0f;
#pragma unroll
                        for (int c = 0; c < VEC; ++c) acc = fmaf(xv[u][c], gv[u][c], acc);
                        d[u] = ok ? acc : 0.0f;
                    }
                }
                if constexpr (!EVEC) {
#pragma unroll
                    for (int off = U / 2; off > 0; off >>= 1) {
                        const bool upper = (sl & off) != 0;
#pragma unroll
                        for (int t = 0; t < off; ++t) {
                            const float give = upper ? d[t] : d[t + off];
                            const float keep = upper ? d[t + off] : d[t];
                            d[t] = keep + __shfl_xor(give, off, LPR);
                        }
                    }
                    float r = d[0];   // position t0 + sl % U, summed over this lane's aligned group of U lanes
#pragma unroll
                    for (int off = U; off < LPR; off <<= 1) r += __shfl_xor(r, off, LPR);
                    if (sl / U == t0 / U) mine += r;
                }
            }
        }
        if constexpr (!EVEC) {
            if (have) grad_e[k_own] = mine;
        }
    }
}

template <int LPR, int VEC>
gnn_status launch_edge_gradient(const gnn_graph *g, int F, bool evec, const float *x, const float *gp,
                                const int32_t *winners, float *grad_e, hipStream_t s, bool csr_out = false)
{
    const int32_t *perm = csr_out ? nullptr : g->perm;
    const int64_t blocks = std::min<int64_t>(gnn_div_up(g->num_edges, kThreads), 256 * 16);
#define GNN_EDGE_GRADIENT(EV, WN)                                                                                   \
    hipLaunchKernelGGL((edge_gradient_kernel<LPR, VEC, EV, WN>), dim3((unsigned)blocks), dim3(kThreads), 0, s, g->rowidx, \
                       g->colidx, perm, g->num_edges, F, x, gp, winners, grad_e)
    if (evec) {
        if (winners) GNN_EDGE_GRADIENT(true, true);
        else GNN_EDGE_GRADIENT(true, false);
    } else {
        if (winners) GNN_EDGE_GRADIENT(false, true);
        else GNN_EDGE_GRADIENT(false, false);
    }
#undef GNN_EDGE_GRADIENT
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

// Per edge (j -> i): <x[j,:], y[i,:]> (or the element-wise product when evec), in the caller's edge
// order or in CSR order.
gnn_status edge_products(const gnn_graph *g, int F, bool evec, const float *x, const float *y, const int32_t *winners,
                         float *out, hipStream_t s, bool csr_out)
{
    const bool vec4 = (F % 4 == 0) && aligned16(x) && aligned16(y) && (!evec || aligned16(out)) && aligned16(winners);
    if (vec4) {
        const int cols = F / 4;
        if (cols <= 4) return launch_edge_gradient<4, 4>(g, F, evec, x, y, winners, out, s, csr_out);
        if (cols <= 8) return launch_edge_gradient<8, 4>(g, F, evec, x, y, winners, out, s, csr_out);
        if (cols <= 16) return launch_edge_gradient<16, 4>(g, F, evec, x, y, winners, out, s, csr_out);
        return launch_edge_gradient<32, 4>(g, F, evec, x, y, winners, out, s, csr_out);
    }
    if (F <= 16) return launch_edge_gradient<16, 1>(g, F, evec, x, y, winners, out, s, csr_out);
    return launch_edge_gradient<64, 1>(g, F, evec, x, y, winners, out, s, csr_out);
}

}  // namespace

gnn_status gnn_launch_edge_dot(const gnn_graph *g, const float *d_x_src, const float *d_y_dst, int32_t feat_dim,
                               float *d_out, gnn_edge_order out_order, void *stream)
{
    if (g->num_edges == 0) return GNN_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (out_order == GNN_EDGE_ORDER_COO && g->route && gnn_aligned16(d_out)) {
        // one scalar per edge: written in CSR order (a stream), moved to the caller's order by the route
        GNN_TRY(edge_products(g, feat_dim, false, d_x_src, d_y_dst, nullptr, g->route->staged, s, true));
        return gnn_route_csr_to_coo(g, g->route->staged, d_out, s);
    }
    return edge_products(g, feat_dim, false, d_x_src, d_y_dst, nullptr, d_out, s, out_order == GNN_EDGE_ORDER_CSR);
}

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
    if (msg == GNN_MSG_XJ_SUB_XI || msg == GNN_MSG_XI_DOT_XJ) return GNN_ERR_UNSUPPORTED;
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
    if (msg == GNN_MSG_XJ_SUB_XI || msg == GNN_MSG_XI_DOT_XJ || aggr == GNN_AGGR_MIN || aggr == GNN_AGGR_PROD)
        return GNN_ERR_UNSUPPORTED;
    if (msg != GNN_MSG_COPY_XJ && msg != GNN_MSG_E_MUL_XJ) return GNN_ERR_BAD_SIZE;
    if (aggr != GNN_AGGR_SUM && aggr != GNN_AGGR_MEAN && aggr != GNN_AGGR_MAX) return GNN_ERR_BAD_SIZE;
    if (aggr == GNN_AGGR_MAX && !d_argmax) return GNN_ERR_NULL;
    if (g->bipartite) return GNN_ERR_UNSUPPORTED;   // one node set only

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
        if (e_dim == 1 && !winners && g->route && gnn_aligned16(d_grad_e)) {
            // one gradient per edge: written in CSR order (a stream) and moved to the caller's order by the route
            GNN_TRY(edge_products(g, F, false, d_x, gp, nullptr, g->route->staged, s, true));
            return gnn_route_csr_to_coo(g, g->route->staged, d_grad_e, s);
        }
        return edge_products(g, F, e_dim != 1, d_x, gp, winners, d_grad_e, s, false);
    }
    return GNN_OK;
}

}  // extern "C"
