// GAT-style attention layer (layer named in the paper, section 3, "Graph Convolutional
// Layers"): an apply_edges step that scores every edge from its two endpoints, a softmax of the
// scores over each destination's neighbourhood, and a weighted-sum aggregation -- fused here
// into one pass over the by-destination CSR so that neither the [E x heads] scores nor the
// attention weights are ever written to memory.
//
//   h = X W (MFMA projection);  sl = <a_src, h> and sr = <a_dst, h> per node and head;
//   per destination row: running (max, denominator, weighted feature sum) per head ("online"
//   softmax), updated a batch of edges at a time -- the batch's largest score joins the maximum,
//   the state is rescaled once, each edge adds exp(score - max) times its slice -- and divided
//   once at the end.
// Work decomposition is the one of propagate: sub-group per short row, wavefront per piece of a
// long row, split rows merged afterwards in piece order.  Partial states (edge slots of a
// wavefront, pieces of a split row) are combined by rescaling each to the common maximum and
// adding.
#include "gnn_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / 64;

struct GatParams {
    const int32_t *rowptr, *colidx;
    const float *h, *sl, *sr;
    const float *a_src;                  // [H x ch]: the source half of the attention vector (score recomputation)
    float *out;
    float *stats;                        // optional [N x H x 2]: (segment maximum, denominator) per row and head
    float *slot_acc, *slot_m, *slot_d;   // [slots x HC] each
    const int32_t *small_rows, *item_row, *item_start, *item_slot, *split_rows, *split_slot0;
    int32_t n_small, n_items, n_split, chunk, HC, H, ch, item_blocks;
    float slope;
};

template <int VEC>
struct State {
    float m, d;
    float acc[VEC];
};

template <int VEC>
__device__ __forceinline__ void state_init(State<VEC> &s)
{
    s.m = -INFINITY;
    s.d = 0.0f;
#pragma unroll
    for (int c = 0; c < VEC; ++c) s.acc[c] = 0.0f;
}

// e^x through the hardware's 2^x: off by at most about (1 + |x|) * 2^-23 of the result.  The weights of a row
// are only ever used as ratios (weighted sum over denominator), and the edge loop below lives on arithmetic:
// the library routine would be a third of its instructions.
__device__ __forceinline__ float exp_hw(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }

// Adds U edges at once to the running softmax-weighted sum: the largest score of the batch joins the running
// maximum first, the state is rescaled to it once, and every edge then costs one exponential and VEC + 1
// multiply-adds.  An edge that is masked off carries the score -inf (weight 0) and a zero slice.
template <int VEC, int U>
__device__ __forceinline__ void state_add_batch(State<VEC> &s, const float (&sc)[U], const float (&hv)[U][VEC])
{
    float bm = sc[0];
#pragma unroll
    for (int u = 1; u < U; ++u) bm = fmaxf(bm, sc[u]);
    const float nm = fmaxf(s.m, bm);
    const float ref = (nm == -INFINITY) ? 0.0f : nm;   // nothing seen so far and nothing valid in the batch
    const float scale = exp_hw(s.m - ref);              // e^-inf = 0 on the first batch, where d and acc are zero
    s.m = nm;
    s.d *= scale;
#pragma unroll
    for (int c = 0; c < VEC; ++c) s.acc[c] *= scale;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float pe = exp_hw(sc[u] - ref);
        s.d += pe;
#pragma unroll
        for (int c = 0; c < VEC; ++c) s.acc[c] = fmaf(pe, hv[u][c], s.acc[c]);
    }
}

// Brings a state to the maximum `m` (not below its own).
template <int VEC>
__device__ __forceinline__ void state_rescale(State<VEC> &s, float m)
{
    const float f = (s.m == -INFINITY) ? 0.0f : expf(s.m - m);
    s.m = m;
    s.d *= f;
#pragma unroll
    for (int c = 0; c < VEC; ++c) s.acc[c] *= f;
}

template <int VEC>
__device__ __forceinline__ void load_vec(float *v, const float *__restrict__ p)
{
    if constexpr (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = *p;
    }
}

template <int VEC>
__device__ __forceinline__ void store_vec(float *__restrict__ p, const float *v)
{
    if constexpr (VEC == 4)
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    else
        *p = v[0];
}

template <int VEC>
__device__ __forceinline__ void write_out(const GatParams &p, int row, int col, const State<VEC> &s)
{
    float v[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) v[c] = s.d > 0.0f ? s.acc[c] / s.d : 0.0f;
    store_vec<VEC>(p.out + (int64_t)row * p.HC + col, v);
    if (p.stats && col % p.ch == 0) {
        float *st = p.stats + ((int64_t)row * p.H + col / p.ch) * 2;
        st[0] = s.m;
        st[1] = s.d;
    }
}

__device__ __forceinline__ float lrelu(float v, float slope) { return v > 0.0f ? v : slope * v; }

// Source half of an edge's score from the gathered feature slice itself: <a_src, h_j> over the head's channels,
// which LPH consecutive lanes hold VEC at a time.  The per-lane partial is an fma chain from zero, the lanes are
// added pairwise (xor 1, 2, ...): the same operations in the same order as node_scores_kernel, so the value is
// bit for bit the stored sl[j, head] -- without the second gather per edge.
template <int VEC, int LPH>
__device__ __forceinline__ float source_score(const float *as, const float *hv)
{
    float part = 0.0f;
#pragma unroll
    for (int c = 0; c < VEC; ++c) part = fmaf(as[c], hv[c], part);
#pragma unroll
    for (int off = 1; off < LPH; off <<= 1) part += __shfl_xor(part, off, 64);
    return part;
}

template <int LPR, int VEC, int LPH>
__device__ __forceinline__ void gat_short_rows(const GatParams &p, int block)
{
    constexpr int NSG = 64 / LPR;
    constexpr int U = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sl_ = lane % LPR, sg = lane / LPR;
    const int64_t sgid = ((int64_t)block * kWavesPerBlock + wave) * NSG + sg;
    const bool have = sgid < p.n_small;
    int row = 0, start = 0, deg = 0;
    if (have) {
        row = p.small_rows[sgid];
        start = p.rowptr[row];
        deg = p.rowptr[row + 1] - start;
    }
    int wmax = deg;
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) wmax = max(wmax, __shfl_xor(wmax, off, 64));

    for (int cb = 0; cb * LPR * VEC < p.HC; ++cb) {
        const int col = (cb * LPR + sl_) * VEC;
        const bool colok = have && col < p.HC;
        const int hd = colok ? col / p.ch : 0;
        const float sr_i = colok ? p.sr[(int64_t)row * p.H + hd] : 0.0f;
        float as[VEC];   // LPH > 0: scores are recomputed from the gathered slices
#pragma unroll
        for (int c = 0; c < VEC; ++c) as[c] = (LPH > 0 && colok) ? p.a_src[col + c] : 0.0f;
        State<VEC> st;
        state_init(st);
        for (int base = 0; base < wmax; base += LPR) {
            int my_j = 0;
            if (base + sl_ < deg) my_j = p.colidx[start + base + sl_];
            const int cnt = min(LPR, wmax - base);
            for (int t0 = 0; t0 < cnt; t0 += U) {
                float hv[U][VEC], sc[U];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int t = t0 + u;
                    const int j = __shfl(my_j, t, LPR);
                    ok[u] = colok && (base + t < deg);
                    sc[u] = 0.0f;
#pragma unroll
                    for (int c = 0; c < VEC; ++c) hv[u][c] = 0.0f;
                    if (ok[u]) {
                        load_vec<VEC>(hv[u], p.h + (int64_t)j * p.HC + col);
                        if constexpr (LPH == 0) sc[u] = p.sl[(int64_t)j * p.H + hd];
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (LPH > 0) sc[u] = source_score<VEC, LPH>(as, hv[u]);
                    sc[u] = ok[u] ? lrelu(sc[u] + sr_i, p.slope) : -INFINITY;
                }
                state_add_batch<VEC, U>(st, sc, hv);
            }
        }
        if (colok) write_out<VEC>(p, row, col, st);
    }
}

template <int LPR, int VEC, int LPH>
__device__ __forceinline__ void gat_long_pieces(const GatParams &p, int block)
{
    constexpr int NSG = 64 / LPR;
    constexpr int U = (LPR >= 4) ? 4 : LPR;   // gathers in flight per lane (measured: 8 is slower)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sl_ = lane % LPR, sg = lane / LPR;
    const int it = block * kWavesPerBlock + wave;
    if (it >= p.n_items) return;
    const int row = p.item_row[it];
    const int start = p.item_start[it];
    const int slot = p.item_slot[it];
    const int end = min(start + p.chunk, p.rowptr[row + 1]);

    for (int cb = 0; cb * LPR * VEC < p.HC; ++cb) {
        const int col = (cb * LPR + sl_) * VEC;
        const bool colok = col < p.HC;
        const int hd = colok ? col / p.ch : 0;
        const float sr_i = colok ? p.sr[(int64_t)row * p.H + hd] : 0.0f;
        float as[VEC];   // LPH > 0: scores are recomputed from the gathered slices
#pragma unroll
        for (int c = 0; c < VEC; ++c) as[c] = (LPH > 0 && colok) ? p.a_src[col + c] : 0.0f;
        State<VEC> st;
        state_init(st);
        for (int base = start; base < end; base += 64) {
            const int n = min(64, end - base);
            int my_j = 0;
            if (lane < n) my_j = p.colidx[base + lane];
            for (int t0 = 0; t0 * NSG < n; t0 += U) {
                float hv[U][VEC], sc[U];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int pos = (t0 + u) * NSG + sg;
                    const int j = __shfl(my_j, pos, 64);
                    ok[u] = colok && pos < n;
                    sc[u] = 0.0f;
#pragma unroll
                    for (int c = 0; c < VEC; ++c) hv[u][c] = 0.0f;
                    if (ok[u]) {
                        load_vec<VEC>(hv[u], p.h + (int64_t)j * p.HC + col);
                        if constexpr (LPH == 0) sc[u] = p.sl[(int64_t)j * p.H + hd];
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if constexpr (LPH > 0) sc[u] = source_score<VEC, LPH>(as, hv[u]);
                    sc[u] = ok[u] ? lrelu(sc[u] + sr_i, p.slope) : -INFINITY;
                }
                state_add_batch<VEC, U>(st, sc, hv);
            }
        }
        // Across the edge slots: the common maximum first (exact in any order), one rescaling per lane, then plain
        // sums, which come out the same in every lane.
        {
            float mm = st.m;
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) mm = fmaxf(mm, __shfl_xor(mm, off, 64));
            state_rescale<VEC>(st, mm);
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) {
                st.d += __shfl_xor(st.d, off, 64);
#pragma unroll
                for (int c = 0; c < VEC; ++c) st.acc[c] += __shfl_xor(st.acc[c], off, 64);
            }
        }
        if (sg == 0 && colok) {
            if (slot < 0) {
                write_out<VEC>(p, row, col, st);
            } else {
                const int64_t q = (int64_t)slot * p.HC + col;
                float mv[VEC], dv[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) { mv[c] = st.m; dv[c] = st.d; }
                store_vec<VEC>(p.slot_acc + q, st.acc);
                store_vec<VEC>(p.slot_m + q, mv);
                store_vec<VEC>(p.slot_d + q, dv);
            }
        }
    }
}

template <int LPR, int VEC, int LPH>
__global__ __launch_bounds__(kThreads) void gat_kernel(const GatParams p)
{
    if ((int)blockIdx.x < p.item_blocks)
        gat_long_pieces<LPR, VEC, LPH>(p, blockIdx.x);
    else
        gat_short_rows<LPR, VEC, LPH>(p, blockIdx.x - p.item_blocks);
}

template <int LPR, int VEC>
__global__ __launch_bounds__(kThreads) void gat_merge_kernel(const GatParams p)
{
    const int64_t s = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / LPR;
    const int sl_ = threadIdx.x % LPR;
    if (s >= p.n_split) return;
    const int row = p.split_rows[s];
    const int slot0 = p.split_slot0[s];
    const int deg = p.rowptr[row + 1] - p.rowptr[row];
    const int pieces = (deg + p.chunk - 1) / p.chunk;
    for (int cb = 0; cb * LPR * VEC < p.HC; ++cb) {
        const int col = (cb * LPR + sl_) * VEC;
        if (col >= p.HC) continue;
        // pieces in piece order: the maximum over the pieces first, then every piece rescaled to it and added
        State<VEC> st;
        state_init(st);
        for (int c = 0; c < pieces; ++c) st.m = fmaxf(st.m, p.slot_m[(int64_t)(slot0 + c) * p.HC + col]);
        for (int c = 0; c < pieces; ++c) {
            const int64_t q = (int64_t)(slot0 + c) * p.HC + col;
            State<VEC> pc;
            pc.m = p.slot_m[q];
            pc.d = p.slot_d[q];
            load_vec<VEC>(pc.acc, p.slot_acc + q);
            state_rescale<VEC>(pc, st.m);
            st.d += pc.d;
#pragma unroll
            for (int k = 0; k < VEC; ++k) st.acc[k] += pc.acc[k];
        }
        write_out<VEC>(p, row, col, st);
    }
}

// sl[i,hd] = <a_src[hd,:], h[i,hd,:]>,  sr[i,hd] = <a_dst[hd,:], h[i,hd,:]>
// One thread per (node, head); with VEC = 4 the head's channels are read as 128-bit pieces.  Order of the
// sum: an fma chain from zero per group of VEC channels; the group sums are added pairwise as a tree when their
// number is a power of two (the order source_score() uses), else one after the other.
template <int VEC>
__global__ __launch_bounds__(kThreads) void node_scores_kernel(const float *__restrict__ h, int64_t N, int H, int ch,
                                                               const float *__restrict__ a_src,
                                                               const float *__restrict__ a_dst,
                                                               float *__restrict__ sl, float *__restrict__ sr)
{
    constexpr int kTreeGroups = 4;
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= N * H) return;
    const int hd = (int)(idx % H);
    const float *hp = h + idx * ch;   // (i*H + hd)*ch
    const int groups = ch / VEC;
    const bool tree = groups <= kTreeGroups && (groups & (groups - 1)) == 0;
    float lt[kTreeGroups] = {0.f, 0.f, 0.f, 0.f}, rt[kTreeGroups] = {0.f, 0.f, 0.f, 0.f};
    float l = 0.0f, r = 0.0f;
    for (int g = 0; g < groups; ++g) {
        float v[VEC];
        load_vec<VEC>(v, hp + g * VEC);
        float lp = 0.0f, rp = 0.0f;
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
            lp = fmaf(a_src[hd * ch + g * VEC + q], v[q], lp);
            rp = fmaf(a_dst[hd * ch + g * VEC + q], v[q], rp);
        }
        if (tree) {
#pragma unroll
            for (int t = 0; t < kTreeGroups; ++t)
                if (t == g) { lt[t] = lp; rt[t] = rp; }
        } else {
            l += lp;
            r += rp;
        }
    }
    if (tree) {
        if (groups == 1) { l = lt[0]; r = rt[0]; }
        else if (groups == 2) { l = lt[0] + lt[1]; r = rt[0] + rt[1]; }
        else { l = (lt[0] + lt[1]) + (lt[2] + lt[3]); r = (rt[0] + rt[1]) + (rt[2] + rt[3]); }
    }
    sl[idx] = l;
    sr[idx] = r;
}

template <int LPR, int VEC>
gnn_status launch_gat(const GatParams &p, hipStream_t stream)
{
    constexpr int NSG = 64 / LPR;
    const int64_t blocks = p.item_blocks + gnn_div_up(p.n_small, kWavesPerBlock * NSG);
    if (blocks > 0) {
        // Heads of 4, 8 or 16 channels (1, 2 or 4 lanes of a 128-bit column group): the source half of the score
        // is recomputed from the gathered slice; other widths gather it from the per-node array.
        const int lph = (VEC == 4 && p.ch % 4 == 0) ? p.ch / 4 : 0;
        const dim3 grid((unsigned)blocks);
        if (VEC == 4 && lph == 1)
            hipLaunchKernelGGL((gat_kernel<LPR, VEC, (VEC == 4 ? 1 : 0)>), grid, dim3(kThreads), 0, stream, p);
        else if (VEC == 4 && lph == 2 && LPR >= 2)
            hipLaunchKernelGGL((gat_kernel<LPR, VEC, (VEC == 4 ? 2 : 0)>), grid, dim3(kThreads), 0, stream, p);
        else if (VEC == 4 && lph == 4 && LPR >= 4)
            hipLaunchKernelGGL((gat_kernel<LPR, VEC, (VEC == 4 ? 4 : 0)>), grid, dim3(kThreads), 0, stream, p);
        else
            hipLaunchKernelGGL((gat_kernel<LPR, VEC, 0>), grid, dim3(kThreads), 0, stream, p);
        GNN_LAUNCH_CHECK();
    }
    if (p.n_split > 0) {
        const int64_t cblocks = gnn_div_up((int64_t)p.n_split * LPR, kThreads);
        hipLaunchKernelGGL((gat_merge_kernel<LPR, VEC>), dim3((unsigned)cblocks), dim3(kThreads), 0, stream, p);
        GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

}  // namespace

gnn_status gnn_launch_node_scores(const float *d_h, int64_t N, int heads, int ch, const float *d_a_src,
                                  const float *d_a_dst, float *d_sl, float *d_sr, hipStream_t s)
{
    const dim3 ns_grid((unsigned)gnn_div_up(N * heads, kThreads));
    if (ch % 4 == 0)
        hipLaunchKernelGGL(node_scores_kernel<4>, ns_grid, dim3(kThreads), 0, s, d_h, N, heads, ch, d_a_src, d_a_dst,
                           d_sl, d_sr);
    else
        hipLaunchKernelGGL(node_scores_kernel<1>, ns_grid, dim3(kThreads), 0, s, d_h, N, heads, ch, d_a_src, d_a_dst,
                           d_sl, d_sr);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

extern "C" {

size_t gnn_gatconv_workspace_bytes(int32_t num_nodes, int32_t heads, int32_t ch)
{
    if (num_nodes <= 0 || heads <= 0 || ch <= 0) return 0;
    return align256((size_t)num_nodes * heads * ch * sizeof(float)) +
           2 * align256((size_t)num_nodes * heads * sizeof(float));
}

gnn_status gnn_gatconv(const gnn_graph *g, const float *d_x, int32_t f_in, const float *d_w, const float *d_a_src,
                       const float *d_a_dst, int32_t heads, int32_t ch, float negative_slope, float *d_out,
                       float *d_softmax_stats, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!g || !d_x || !d_w || !d_a_src || !d_a_dst || !d_out || !d_workspace) return GNN_ERR_NULL;
    if (f_in <= 0 || heads <= 0 || ch <= 0) return GNN_ERR_BAD_SIZE;
    if (g->bipartite) return GNN_ERR_UNSUPPORTED;   // one node set only
    const int32_t N = g->num_nodes;
    if (workspace_bytes < gnn_gatconv_workspace_bytes(N, heads, ch)) return GNN_ERR_BAD_SIZE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255u) return GNN_ERR_BAD_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int HC = heads * ch;
    char *ws = static_cast<char *>(d_workspace);
    float *h = reinterpret_cast<float *>(ws);
    float *sl = reinterpret_cast<float *>(ws + align256((size_t)N * HC * sizeof(float)));
    float *sr = reinterpret_cast<float *>(ws + align256((size_t)N * HC * sizeof(float)) +
                                          align256((size_t)N * heads * sizeof(float)));

    GNN_TRY(gnn_dense_xw(d_x, N, f_in, d_w, HC, nullptr, h, stream));
    GNN_TRY(gnn_launch_node_scores(h, N, heads, ch, d_a_src, d_a_dst, sl, sr, s));

    GatParams p{};
    p.rowptr = g->rowptr; p.colidx = g->colidx;
    p.h = h; p.sl = sl; p.sr = sr; p.a_src = d_a_src; p.out = d_out; p.stats = d_softmax_stats;
    p.small_rows = g->small_rows; p.item_row = g->item_row; p.item_start = g->item_start;
    p.item_slot = g->item_slot; p.split_rows = g->split_rows; p.split_slot0 = g->split_slot0;
    p.n_small = g->n_small; p.n_items = g->n_items; p.n_split = g->n_split; p.chunk = g->chunk;
    p.HC = HC; p.H = heads; p.ch = ch; p.slope = negative_slope;
    p.item_blocks = (int32_t)gnn_div_up(g->n_items, kWavesPerBlock);
    if (g->n_slots > 0) {
        float *scratch = nullptr;
        GNN_TRY(gnn_graph_scratch(g, 3 * (size_t)g->n_slots * HC, &scratch));
        p.slot_acc = scratch;
        p.slot_m = scratch + (size_t)g->n_slots * HC;
        p.slot_d = scratch + 2 * (size_t)g->n_slots * HC;
    }
    const bool vec4 = (ch % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_out) & 15u) == 0);
    if (vec4) {
        const int cols = HC / 4;
        if (cols <= 8) return launch_gat<8, 4>(p, s);
        if (cols <= 16) return launch_gat<16, 4>(p, s);
        if (cols <= 32) return launch_gat<32, 4>(p, s);
        return launch_gat<64, 4>(p, s);
    }
    if (HC <= 16) return launch_gat<16, 1>(p, s);
    return launch_gat<64, 1>(p, s);
}

}  // extern "C"
