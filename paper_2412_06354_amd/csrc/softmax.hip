// Segment softmax: softmax over each destination node's incoming edges, per head -- the
// normalisation attention layers apply to per-edge scores (GAT is named in the paper,
// section 3, "Graph Convolutional Layers"; a per-edge score is an apply_edges result and
// the normalisation is a reduction over each neighbourhood followed by a per-edge rescale).
//
// Two phases over the by-destination CSR:
//   1. per (row, head) statistics  m = max of the scores, den = sum exp(score - m):
//      short rows: one thread per (row, head);
//      long rows : one wavefront per piece of <= chunk edges, lanes = (edge slot, head),
//                  xor-shuffle reductions; pieces of a split row are merged in piece order;
//   2. one thread per (edge, head):  out = exp(score - m[row]) / den[row]   (perfectly balanced).
#include "gnn_internal.h"

namespace {

constexpr int kThreads = 256;

struct SmParams {
    const int32_t *rowptr, *perm, *rowidx;
    const float *s;
    float *out;
    float2 *rowstat;    // [N x H]  (m, den)
    float2 *slotstat;   // [slots x H]
    const int32_t *small_rows, *item_row, *item_start, *item_slot, *split_rows, *split_slot0;
    int32_t n_small, n_items, n_split, chunk, H, coo;
    int64_t E;
};

__global__ __launch_bounds__(kThreads) void stats_short_kernel(const SmParams p)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t ri = idx / p.H;
    const int h = (int)(idx - ri * p.H);
    if (ri >= p.n_small) return;
    const int row = p.small_rows[ri];
    const int start = p.rowptr[row], end = p.rowptr[row + 1];
    float m = -INFINITY;
    for (int q = start; q < end; ++q) {
        const int64_t eid = p.coo ? p.perm[q] : q;
        m = fmaxf(m, p.s[eid * p.H + h]);
    }
    float den = 0.0f;
    for (int q = start; q < end; ++q) {
        const int64_t eid = p.coo ? p.perm[q] : q;
        den += expf(p.s[eid * p.H + h] - m);
    }
    p.rowstat[(int64_t)row * p.H + h] = make_float2(m, den);
}

template <int HP /* heads per pass, power of two <= 64 */>
__global__ __launch_bounds__(kThreads) void stats_long_kernel(const SmParams p)
{
    constexpr int ES = 64 / HP;   // edges per step
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int it = blockIdx.x * (kThreads / 64) + wave;
    if (it >= p.n_items) return;
    const int row = p.item_row[it];
    const int start = p.item_start[it];
    const int slot = p.item_slot[it];
    const int end = min(start + p.chunk, p.rowptr[row + 1]);
    const int hl = lane % HP, es = lane / HP;
    for (int hb = 0; hb < p.H; hb += HP) {
        const int h = hb + hl;
        const bool hok = h < p.H;
        float m = -INFINITY;
        for (int q = start + es; q < end; q += ES) {
            const int64_t eid = p.coo ? p.perm[q] : q;
            if (hok) m = fmaxf(m, p.s[eid * p.H + h]);
        }
#pragma unroll
        for (int off = HP; off < 64; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        float den = 0.0f;
        for (int q = start + es; q < end; q += ES) {
            const int64_t eid = p.coo ? p.perm[q] : q;
            if (hok) den += expf(p.s[eid * p.H + h] - m);
        }
#pragma unroll
        for (int off = HP; off < 64; off <<= 1) den += __shfl_xor(den, off, 64);
        if (es == 0 && hok) {
            if (slot < 0)
                p.rowstat[(int64_t)row * p.H + h] = make_float2(m, den);
            else
                p.slotstat[(int64_t)slot * p.H + h] = make_float2(m, den);
        }
    }
}

__global__ __launch_bounds__(kThreads) void stats_merge_kernel(const SmParams p)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t si = idx / p.H;
    const int h = (int)(idx - si * p.H);
    if (si >= p.n_split) return;
    const int row = p.split_rows[si];
    const int slot0 = p.split_slot0[si];
    const int deg = p.rowptr[row + 1] - p.rowptr[row];
    const int pieces = (deg + p.chunk - 1) / p.chunk;
    float m = -INFINITY;
    for (int c = 0; c < pieces; ++c) m = fmaxf(m, p.slotstat[(int64_t)(slot0 + c) * p.H + h].x);
    float den = 0.0f;
    for (int c = 0; c < pieces; ++c) {
        const float2 st = p.slotstat[(int64_t)(slot0 + c) * p.H + h];
        den += st.y * expf(st.x - m);
    }
    p.rowstat[(int64_t)row * p.H + h] = make_float2(m, den);
}

__global__ __launch_bounds__(kThreads) void normalise_kernel(const SmParams p)
{
    const int64_t total = p.E * p.H;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total; idx += stride) {
        const int64_t q = idx / p.H;
        const int h = (int)(idx - q * p.H);
        const int row = p.rowidx[q];
        const int64_t eid = p.coo ? p.perm[q] : q;
        const float2 st = p.rowstat[(int64_t)row * p.H + h];
        p.out[eid * p.H + h] = expf(p.s[eid * p.H + h] - st.x) / st.y;
    }
}

}  // namespace

extern "C" gnn_status gnn_segment_softmax(const gnn_graph *g, const float *d_scores, int32_t heads,
                                          gnn_edge_order order, float *d_out, void *stream)
{
    if (!g) return GNN_ERR_NULL;
    if (heads <= 0) return GNN_ERR_BAD_SIZE;
    if (order != GNN_EDGE_ORDER_COO && order != GNN_EDGE_ORDER_CSR) return GNN_ERR_BAD_SIZE;
    if (g->num_edges == 0) return GNN_OK;
    if (!d_scores || !d_out) return GNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t stat_floats = 2 * ((size_t)g->num_nodes + (size_t)g->n_slots) * heads;
    GNN_TRY(gnn_graph_reserve_scratch(g, stat_floats));

    SmParams p{};
    p.rowptr = g->rowptr; p.perm = g->perm; p.rowidx = g->rowidx;
    p.s = d_scores; p.out = d_out;
    p.rowstat = reinterpret_cast<float2 *>(g->scratch);
    p.slotstat = p.rowstat + (size_t)g->num_nodes * heads;
    p.small_rows = g->small_rows; p.item_row = g->item_row; p.item_start = g->item_start;
    p.item_slot = g->item_slot; p.split_rows = g->split_rows; p.split_slot0 = g->split_slot0;
    p.n_small = g->n_small; p.n_items = g->n_items; p.n_split = g->n_split; p.chunk = g->chunk;
    p.H = heads; p.coo = (order == GNN_EDGE_ORDER_COO) ? 1 : 0; p.E = g->num_edges;

    if (g->n_items > 0) {
        const unsigned blocks = (unsigned)gnn_div_up(g->n_items, kThreads / 64);
        int hp = 1;
        while (hp < heads && hp < 64) hp <<= 1;
        switch (hp) {
        case 1: hipLaunchKernelGGL(stats_long_kernel<1>, dim3(blocks), dim3(kThreads), 0, s, p); break;
        case 2: hipLaunchKernelGGL(stats_long_kernel<2>, dim3(blocks), dim3(kThreads), 0, s, p); break;
        case 4: hipLaunchKernelGGL(stats_long_kernel<4>, dim3(blocks), dim3(kThreads), 0, s, p); break;
        case 8: hipLaunchKernelGGL(stats_long_kernel<8>, dim3(blocks), dim3(kThreads), 0, s, p); break;
        case 16: hipLaunchKernelGGL(stats_long_kernel<16>, dim3(blocks), dim3(kThreads), 0, s, p); break;
        case 32: hipLaunchKernelGGL(stats_long_kernel<32>, dim3(blocks), dim3(kThreads), 0, s, p); break;
        default: hipLaunchKernelGGL(stats_long_kernel<64>, dim3(blocks), dim3(kThreads), 0, s, p); break;
        }
        GNN_LAUNCH_CHECK();
    }
    if (g->n_small > 0) {
        const unsigned blocks = (unsigned)gnn_div_up((int64_t)g->n_small * heads, kThreads);
        hipLaunchKernelGGL(stats_short_kernel, dim3(blocks), dim3(kThreads), 0, s, p);
        GNN_LAUNCH_CHECK();
    }
    if (g->n_split > 0) {
        const unsigned blocks = (unsigned)gnn_div_up((int64_t)g->n_split * heads, kThreads);
        hipLaunchKernelGGL(stats_merge_kernel, dim3(blocks), dim3(kThreads), 0, s, p);
        GNN_LAUNCH_CHECK();
    }
    {
        const int64_t total = g->num_edges * heads;
        const unsigned blocks = (unsigned)std::min<int64_t>(gnn_div_up(total, kThreads), 256 * 256);
        hipLaunchKernelGGL(normalise_kernel, dim3(blocks), dim3(kThreads), 0, s, p);
        GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
}
