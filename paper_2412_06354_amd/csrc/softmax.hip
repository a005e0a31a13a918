// Segment softmax: softmax over each destination node's incoming edges, per head -- the
// normalisation attention layers apply to per-edge scores (GAT is named in the paper,
// section 3, "Graph Convolutional Layers"; a per-edge score is an apply_edges result and
// the normalisation is a reduction over each neighbourhood followed by a per-edge rescale).
//
// Two phases:
//   1. per (row, head) statistics  m = max of the scores, den = sum exp(score - m), over the
//      by-destination CSR with the propagate work decomposition: a sub-group of HP lanes per short
//      row, a wavefront per piece of a long row with lanes = (edge slot, head group); a lane owns
//      one head, or four consecutive heads read with one 128-bit load;
//      edge ids are fetched in batches and the score loads of a batch are independent; the
//      running (m, den) pair is updated edge by edge; the lanes of a head group, and the pieces of
//      a split row, are combined by taking the common maximum first and adding the denominators
//      rescaled to it (one exponential per lane or piece);
//   2. one thread per (edge, head), in the order the scores are stored in (so reads and writes
//      stream):  out = exp(score - m[row]) / den[row], the row coming from the stored copy of the
//      destination array (caller's order) or from the sorted destinations (CSR order).
#include "gnn_internal.h"

#include <algorithm>

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / 64;

struct SmParams {
    const int32_t *rowptr, *perm, *row_of_edge;
    const float *s;
    const float *s2;    // backward only: dL/d alpha (s then holds alpha)
    float *out;
    float2 *rowstat;    // [N x H]  (m, den)
    float2 *slotstat;   // [slots x H]
    const int32_t *small_rows, *item_row, *item_start, *item_slot, *split_rows, *split_slot0;
    int32_t n_small, n_items, n_split, chunk, H, coo, item_blocks;
    int64_t E;
};

// (m, d) <- (m, d) + one score v
__device__ __forceinline__ void online_add(float &m, float &d, bool ok, float v)
{
    const float delta = v - m;
    const float e = __expf(-fabsf(delta));     // exp(-inf) = 0 covers the first score (m = -inf)
    const bool up = delta > 0.0f;
    if (ok) {
        d = up ? d * e + 1.0f : d + e;
        m = up ? v : m;
    }
}

// Forward: running (max, denominator).  Backward: d accumulates alpha * dalpha (m is unused).
template <bool BWD>
__device__ __forceinline__ void acc_add(float &m, float &d, bool ok, float v, float w)
{
    if constexpr (BWD) d += ok ? v * w : 0.0f;
    else online_add(m, d, ok, v);
}

template <int HV>
__device__ __forceinline__ void load_heads(float (&v)[HV], const float *__restrict__ p)
{
    if constexpr (HV == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = *p;
    }
}

template <int HV>
__device__ __forceinline__ void store_stats(float2 *__restrict__ dst, const float (&m)[HV], const float (&d)[HV])
{
    if constexpr (HV == 4) {
        float4 *q = reinterpret_cast<float4 *>(dst);
        q[0] = make_float4(m[0], d[0], m[1], d[1]);
        q[1] = make_float4(m[2], d[2], m[3], d[3]);
    } else {
        dst[0] = make_float2(m[0], d[0]);
    }
}

// HP lanes per edge, each lane owns HV consecutive heads (HV = 4: 128-bit score loads).
template <int HP, int HV, bool BWD>
__device__ __forceinline__ void stats_short_rows(const SmParams &p, int block)
{
    constexpr int NSG = 64 / HP;
    constexpr int U = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hl = lane % HP, sg = lane / HP;
    const int64_t sgid = ((int64_t)block * kWavesPerBlock + wave) * NSG + sg;
    const bool have = sgid < p.n_small;
    int row = 0, start = 0, deg = 0;
    if (have) {
        row = p.small_rows[sgid];
        start = p.rowptr[row];
        deg = p.rowptr[row + 1] - start;
    }
    for (int hb = 0; hb < p.H; hb += HP * HV) {
        const int h = hb + hl * HV;
        const bool hok = have && h < p.H;
        float m[HV], d[HV];
#pragma unroll
        for (int c = 0; c < HV; ++c) { m[c] = -INFINITY; d[c] = 0.0f; }
        // U edges at a time, every lane fetching the edge ids it needs itself (the lanes of a sub-group ask for the
        // same word): all U score loads of a step are independent and none of them is masked off by the sub-group width.
        for (int t0 = 0; t0 < deg; t0 += U) {
            float v[U][HV], w[U][HV];
            bool ok[U];
            int64_t at[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = start + t0 + u;
                ok[u] = hok && (t0 + u < deg);
                int eid = 0;
                if (ok[u]) eid = p.coo ? __builtin_nontemporal_load(p.perm + q) : q;
                at[u] = (int64_t)eid * p.H + h;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int c = 0; c < HV; ++c) { v[u][c] = 0.0f; w[u][c] = 0.0f; }
                if (ok[u]) {
                    load_heads<HV>(v[u], p.s + at[u]);
                    if constexpr (BWD) load_heads<HV>(w[u], p.s2 + at[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < HV; ++c) acc_add<BWD>(m[c], d[c], ok[u], v[u][c], w[u][c]);
        }
        if (hok) store_stats<HV>(p.rowstat + (int64_t)row * p.H + h, m, d);
    }
}

template <int HP, int HV, bool BWD>
__device__ __forceinline__ void stats_long_pieces(const SmParams &p, int block)
{
    constexpr int ES = 64 / HP;   // edges per step
    constexpr int U = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int it = block * kWavesPerBlock + wave;
    if (it >= p.n_items) return;   // whole wavefront leaves together
    const int row = p.item_row[it];
    const int start = p.item_start[it];
    const int slot = p.item_slot[it];
    const int end = min(start + p.chunk, p.rowptr[row + 1]);
    const int hl = lane % HP, es = lane / HP;
    for (int hb = 0; hb < p.H; hb += HP * HV) {
        const int h = hb + hl * HV;
        const bool hok = h < p.H;
        float m[HV], d[HV];
#pragma unroll
        for (int c = 0; c < HV; ++c) { m[c] = -INFINITY; d[c] = 0.0f; }
        for (int q0 = start; q0 < end; q0 += ES * U) {
            int eid[U];
            float v[U][HV], w[U][HV];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = q0 + u * ES + es;
                ok[u] = hok && q < end;
                eid[u] = 0;
                if (ok[u]) eid[u] = p.coo ? __builtin_nontemporal_load(p.perm + q) : q;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int c = 0; c < HV; ++c) { v[u][c] = 0.0f; w[u][c] = 0.0f; }
                if (ok[u]) {
                    load_heads<HV>(v[u], p.s + (int64_t)eid[u] * p.H + h);
                    if constexpr (BWD) load_heads<HV>(w[u], p.s2 + (int64_t)eid[u] * p.H + h);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (q0 + u * ES < end) {   // the same for the whole wavefront: an empty step costs no arithmetic
#pragma unroll
                    for (int c = 0; c < HV; ++c) acc_add<BWD>(m[c], d[c], ok[u], v[u][c], w[u][c]);
                }
            }
        }
        // Across the edge slots of a head group.  Forward: the common maximum first (exact in any order), then every
        // lane rescales its denominator once and the denominators are added -- one exponential per lane where a
        // butterfly of pair merges would take two per step, and that arithmetic is what short pieces spend their time on.
        if constexpr (!BWD) {
            float mm[HV];
#pragma unroll
            for (int c = 0; c < HV; ++c) mm[c] = m[c];
#pragma unroll
            for (int off = HP; off < 64; off <<= 1) {
#pragma unroll
                for (int c = 0; c < HV; ++c) mm[c] = fmaxf(mm[c], __shfl_xor(mm[c], off, 64));
            }
#pragma unroll
            for (int c = 0; c < HV; ++c) {
                d[c] = (m[c] == -INFINITY) ? 0.0f : d[c] * expf(m[c] - mm[c]);
                m[c] = mm[c];
            }
        }
#pragma unroll
        for (int off = HP; off < 64; off <<= 1) {
#pragma unroll
            for (int c = 0; c < HV; ++c) d[c] += __shfl_xor(d[c], off, 64);
        }
        if (es == 0 && hok)
            store_stats<HV>((slot < 0 ? p.rowstat + (int64_t)row * p.H : p.slotstat + (int64_t)slot * p.H) + h, m, d);
    }
}

template <int HP, int HV, bool BWD>
__global__ __launch_bounds__(kThreads) void stats_kernel(const SmParams p)
{
    if ((int)blockIdx.x < p.item_blocks)
        stats_long_pieces<HP, HV, BWD>(p, blockIdx.x);
    else
        stats_short_rows<HP, HV, BWD>(p, blockIdx.x - p.item_blocks);
}

// A wavefront per (split row, head): lanes take the row's pieces, a butterfly combines the lanes.  Forward: the
// maximum over the pieces first, then the sum of the denominators rescaled to it; sums of a butterfly are the same
// in every lane (addition commutes), so any lane may store.
template <bool BWD>
__global__ __launch_bounds__(kThreads) void stats_merge_kernel(const SmParams p)
{
    const int lane = threadIdx.x & 63;
    const int64_t idx = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const int64_t si = idx / p.H;
    const int h = (int)(idx - si * p.H);
    if (si >= p.n_split) return;   // whole wavefront leaves together
    const int row = p.split_rows[si];
    const int deg = p.rowptr[row + 1] - p.rowptr[row];
    const int pieces = (deg + p.chunk - 1) / p.chunk;
    const float2 *st = p.slotstat + (int64_t)p.split_slot0[si] * p.H + h;
    float m = -INFINITY, d = 0.0f;
    if constexpr (!BWD) {
        for (int c = lane; c < pieces; c += 64) m = fmaxf(m, st[(int64_t)c * p.H].x);
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        for (int c = lane; c < pieces; c += 64) {
            const float2 q = st[(int64_t)c * p.H];
            d += (q.x == -INFINITY) ? 0.0f : q.y * expf(q.x - m);
        }
    } else {
        for (int c = lane; c < pieces; c += 64) d += st[(int64_t)c * p.H].y;
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) d += __shfl_xor(d, off, 64);
    if (lane == 0) p.rowstat[(int64_t)row * p.H + h] = make_float2(m, d);
}

// The element-wise second phase.  Position k of the score array belongs to row row_of_edge[k]; scores and results
// stream.  A thread handles HV consecutive heads of one edge; a block step covers as many whole edges as its threads
// hold, so a thread's head group never changes and nothing is divided per element.
__host__ __device__ inline int edges_per_block_step(int head_groups)
{
    return head_groups >= kThreads ? 1 : kThreads / head_groups;
}

// FN(k, h, st): k = edge position, h = first head of the group, st = the (m, den) records of (row, h ..).
template <int HV, class FN>
__device__ __forceinline__ void for_each_edge_head_group(const SmParams &p, FN fn)
{
    const int hg = p.H / HV;
    const int epb = edges_per_block_step(hg);
    const int el = (int)threadIdx.x / hg, h0 = (int)threadIdx.x - el * hg;
    if (el >= epb) return;
    for (int64_t k = (int64_t)blockIdx.x * epb + el; k < p.E; k += (int64_t)gridDim.x * epb) {
        const int row = __builtin_nontemporal_load(p.row_of_edge + k);
        // one trip, unless an edge has more head groups than the block has threads
        for (int g = h0; g < hg; g += kThreads) fn(k, g * HV, p.rowstat + (int64_t)row * p.H + g * HV);
    }
}

template <int HV>
__global__ __launch_bounds__(kThreads) void normalise_kernel(const SmParams p)
{
    for_each_edge_head_group<HV>(p, [&](int64_t k, int h, const float2 *st) {
        if constexpr (HV == 4) {
            typedef float v4f __attribute__((ext_vector_type(4)));
            const float4 s0 = reinterpret_cast<const float4 *>(st)[0], s1 = reinterpret_cast<const float4 *>(st)[1];
            const v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p.s + k * p.H + h));
            v4f o = {expf(v.x - s0.x) / s0.y, expf(v.y - s0.z) / s0.w, expf(v.z - s1.x) / s1.y, expf(v.w - s1.z) / s1.w};
            __builtin_nontemporal_store(o, reinterpret_cast<v4f *>(p.out + k * p.H + h));
        } else {
            const float2 q = st[0];
            const float v = __builtin_nontemporal_load(p.s + k * p.H + h);
            __builtin_nontemporal_store(expf(v - q.x) / q.y, p.out + k * p.H + h);
        }
    });
}

// Backward: gs = alpha * (dalpha - t[row]) with t = the row's sum of alpha * dalpha (rowstat.y).
template <int HV>
__global__ __launch_bounds__(kThreads) void jacobian_kernel(const SmParams p)
{
    for_each_edge_head_group<HV>(p, [&](int64_t k, int h, const float2 *st) {
        if constexpr (HV == 4) {
            typedef float v4f __attribute__((ext_vector_type(4)));
            const float4 s0 = reinterpret_cast<const float4 *>(st)[0], s1 = reinterpret_cast<const float4 *>(st)[1];
            const v4f a = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p.s + k * p.H + h));
            const v4f g = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p.s2 + k * p.H + h));
            v4f o = {a.x * (g.x - s0.y), a.y * (g.y - s0.w), a.z * (g.z - s1.y), a.w * (g.w - s1.w)};
            __builtin_nontemporal_store(o, reinterpret_cast<v4f *>(p.out + k * p.H + h));
        } else {
            const float a = __builtin_nontemporal_load(p.s + k * p.H + h);
            const float g = __builtin_nontemporal_load(p.s2 + k * p.H + h);
            __builtin_nontemporal_store(a * (g - st[0].y), p.out + k * p.H + h);
        }
    });
}

template <int HP, int HV, bool BWD>
gnn_status launch_stats(const SmParams &p, hipStream_t s)
{
    const int64_t blocks = p.item_blocks + gnn_div_up(p.n_small, kWavesPerBlock * (64 / HP));
    if (blocks > 0) {
        hipLaunchKernelGGL((stats_kernel<HP, HV, BWD>), dim3((unsigned)blocks), dim3(kThreads), 0, s, p);
        GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
}

template <int HV, bool BWD>
gnn_status launch_stats_hv(const SmParams &p, int lanes_needed, hipStream_t s)
{
    int hp = 1;
    while (hp < lanes_needed && hp < 64) hp <<= 1;
    switch (hp) {
    case 1: return launch_stats<1, HV, BWD>(p, s);
    case 2: return launch_stats<2, HV, BWD>(p, s);
    case 4: return launch_stats<4, HV, BWD>(p, s);
    case 8: return launch_stats<8, HV, BWD>(p, s);
    case 16: return launch_stats<16, HV, BWD>(p, s);
    case 32: return launch_stats<32, HV, BWD>(p, s);
    default: return launch_stats<64, HV, BWD>(p, s);
    }
}

template <bool BWD>
gnn_status run_softmax(const gnn_graph *g, const float *d_in, const float *d_in2, int32_t heads, gnn_edge_order order,
                       float *d_out, void *stream)
{
    if (!g) return GNN_ERR_NULL;
    if (heads <= 0) return GNN_ERR_BAD_SIZE;
    if (order != GNN_EDGE_ORDER_COO && order != GNN_EDGE_ORDER_CSR) return GNN_ERR_BAD_SIZE;
    if (g->num_edges == 0) return GNN_OK;
    if (!d_in || !d_out || (BWD && !d_in2)) return GNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (heads == 1 && order == GNN_EDGE_ORDER_COO && g->route && gnn_aligned16(d_in) && gnn_aligned16(d_out) &&
        (!BWD || gnn_aligned16(d_in2))) {
        // One score per edge in the caller's order: a gather through perm would cost a memory line per edge.  With an
        // edge route the inputs are moved to CSR order in streams (the second one of the backward into the output
        // array, which is free until the end), the CSR-ordered kernels run in place on the route's staging buffer
        // (element-wise: every thread reads its own element before it writes it), and the result is moved back.
        float *staged = g->route->staged;
        GNN_TRY(gnn_route_coo_to_csr(g, d_in, staged, s));
        if (BWD) GNN_TRY(gnn_route_coo_to_csr(g, d_in2, d_out, s));
        GNN_TRY((run_softmax<BWD>(g, staged, BWD ? d_out : nullptr, 1, GNN_EDGE_ORDER_CSR, staged, stream)));
        return gnn_route_csr_to_coo(g, staged, d_out, s);
    }
    const size_t stat_floats = 2 * ((size_t)g->num_nodes + (size_t)g->n_slots) * heads;
    float *scratch = nullptr;
    GNN_TRY(gnn_graph_scratch(g, stat_floats, &scratch));

    SmParams p{};
    p.coo = (order == GNN_EDGE_ORDER_COO) ? 1 : 0;
    p.rowptr = g->rowptr; p.perm = g->perm;
    p.row_of_edge = p.coo ? g->dst_coo : g->rowidx;
    p.s = d_in; p.s2 = d_in2; p.out = d_out;
    p.rowstat = reinterpret_cast<float2 *>(scratch);
    p.slotstat = p.rowstat + (size_t)g->num_nodes * heads;
    p.small_rows = g->small_rows; p.item_row = g->item_row; p.item_start = g->item_start;
    p.item_slot = g->item_slot; p.split_rows = g->split_rows; p.split_slot0 = g->split_slot0;
    p.n_small = g->n_small; p.n_items = g->n_items; p.n_split = g->n_split; p.chunk = g->chunk;
    p.H = heads; p.E = g->num_edges;
    p.item_blocks = (int32_t)gnn_div_up(g->n_items, kWavesPerBlock);

    const bool vec4 = (heads % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_in) & 15u) == 0) &&
                      ((reinterpret_cast<uintptr_t>(d_out) & 15u) == 0) &&
                      ((reinterpret_cast<uintptr_t>(d_in2) & 15u) == 0);
    if (vec4)
        GNN_TRY((launch_stats_hv<4, BWD>(p, heads / 4, s)));
    else
        GNN_TRY((launch_stats_hv<1, BWD>(p, heads, s)));
    if (g->n_split > 0) {
        const unsigned blocks = (unsigned)gnn_div_up((int64_t)g->n_split * heads, kWavesPerBlock);
        hipLaunchKernelGGL(stats_merge_kernel<BWD>, dim3(blocks), dim3(kThreads), 0, s, p);
        GNN_LAUNCH_CHECK();
    }
    {
        const int epb = edges_per_block_step(vec4 ? heads / 4 : heads);
        const unsigned blocks = (unsigned)std::min<int64_t>(gnn_div_up(g->num_edges, epb), 256 * 64);
        if (BWD) {
            if (vec4)
                hipLaunchKernelGGL(jacobian_kernel<4>, dim3(blocks), dim3(kThreads), 0, s, p);
            else
                hipLaunchKernelGGL(jacobian_kernel<1>, dim3(blocks), dim3(kThreads), 0, s, p);
        } else {
            if (vec4)
                hipLaunchKernelGGL(normalise_kernel<4>, dim3(blocks), dim3(kThreads), 0, s, p);
            else
                hipLaunchKernelGGL(normalise_kernel<1>, dim3(blocks), dim3(kThreads), 0, s, p);
        }
        GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
}

}  // namespace

extern "C" gnn_status gnn_segment_softmax(const gnn_graph *g, const float *d_scores, int32_t heads,
                                          gnn_edge_order order, float *d_out, void *stream)
{
    return run_softmax<false>(g, d_scores, nullptr, heads, order, d_out, stream);
}

extern "C" gnn_status gnn_segment_softmax_backward(const gnn_graph *g, const float *d_alpha, const float *d_grad_alpha,
                                                   int32_t heads, gnn_edge_order order, float *d_grad_scores,
                                                   void *stream)
{
    return run_softmax<true>(g, d_alpha, d_grad_alpha, heads, order, d_grad_scores, stream);
}
