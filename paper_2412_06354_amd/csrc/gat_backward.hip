// Backward of the attention layer (the paper's purpose is training: its example differentiates
// through the layers, section 3 "Training Example"; the layer is named in section 3, "Graph
// Convolutional Layers").  With G = dL/d out, per edge k = (j -> i) and head hd:
//     v = sl[j] + sr[i],  alpha = exp(lrelu(v) - max_i) / denominator_i         (recomputed, never stored)
//     dalpha = <G[i,hd,:], h[j,hd,:]>
//     dv = alpha * (dalpha - t[i]) * lrelu'(v),      t[i] = <G[i,hd,:], out[i,hd,:]> = sum_k alpha dalpha
//     dsr[i] = sum over incoming edges of dv,        dsl[j] = sum over outgoing edges of dv
//     dh[j]  = sum over outgoing edges of alpha * G[i]  +  dsl[j] a_src  +  dsr[j] a_dst
//     d a_src = sum_j dsl[j] h[j],  d a_dst = sum_i dsr[i] h[i],  dW = X^T dh,  dX = dh W^T.
// Everything an edge needs can be recomputed from per-node records, so nothing of size [E x heads] is
// ever stored: one pass over the by-destination graph (row i owns G[i] and its record, gathers h[j] and
// sl[j]) yields dsr, one pass over the by-source graph (row j owns h[j] and sl[j], gathers G[i] and the
// 16-byte record (sr, max, 1/denominator, t) of i) yields dsl and the first term of dh.  Both passes are
// plain sums, use the work decomposition of propagate (sub-group per short row, wavefront per piece of a
// long row, split rows merged in piece order) and no atomics: gradients are bitwise reproducible.
// The segment maxima and denominators come from the forward call (its optional statistics output).
#include "gnn_internal.h"

#include <algorithm>

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / 64;

struct GatBwdParams {
    const int32_t *rowptr, *colidx;      // the graph this pass walks (by destination or by source)
    const float *own_vec, *nbr_vec;      // [N x HC]: by destination G / h, by source h / G
    const float *sl;                     // [N x H]
    const float *a_src;                  // [H x ch] (by destination: sl[j] recomputed from the gathered h[j])
    const float4 *rec;                   // [N x H]: (sr, segment maximum, 1 / denominator, t)
    const float *a_dst, *term_dsr;       // by-source pass: the rows it writes also take the score terms
                                         // dsl a_src + dsr a_dst (term_dsr = the by-destination pass's result)
    float *out_vec;                      // [N x HC], by-source pass only
    float *out_s;                        // [N x H]
    float *slot_vec, *slot_s;            // [slots x HC] each
    const int32_t *small_rows, *item_row, *item_start, *item_slot, *split_rows, *split_slot0;
    int32_t n_small, n_items, n_split, chunk, HC, H, ch, lh, item_blocks;
    int32_t lh_pow2;   // lh is a power of two: a head's lanes are combined by an xor tree, else by a loop over them
    int32_t pass_lanes;   // lanes of a row's sub-group that hold columns in one pass over the row: all of them, or
                          // (lh no power of two) the largest multiple of lh, so that no head straddles two passes
    float slope;
};

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

// e^x through the hardware's 2^x (off by at most about (1 + |x|) * 2^-23 of the result): the edge passes live on
// arithmetic, and the library routine would be a fifth of their instructions.
__device__ __forceinline__ float exp_hw(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896341f); }

// What a lane keeps of its own row, and what it accumulates.
template <int VEC>
struct Lane {
    float own[VEC];
    float own_sl;      // by source
    float as[VEC];     // by destination, recomputing: this lane's slice of a_src
    float4 own_rec;    // by destination
    int head_first;    // first lane of this lane's head (heads whose lane count is no power of two)
    float acc_s;
    float acc_v[VEC];  // by source
};

template <int VEC, bool BY_SRC, bool RECOMP>
__device__ __forceinline__ void lane_init(Lane<VEC> &ln, const GatBwdParams &p, bool colok, int row, int col, int hd)
{
#pragma unroll
    for (int c = 0; c < VEC; ++c) ln.as[c] = (RECOMP && colok) ? p.a_src[col + c] : 0.0f;
    ln.own_sl = 0.0f;
    ln.own_rec = make_float4(0.f, 0.f, 0.f, 0.f);
    ln.head_first = max(0, (int)(threadIdx.x & 63) - (col % p.ch) / VEC);
    ln.acc_s = 0.0f;
#pragma unroll
    for (int c = 0; c < VEC; ++c) { ln.own[c] = 0.0f; ln.acc_v[c] = 0.0f; }
    if (colok) {
        load_vec<VEC>(ln.own, p.own_vec + (int64_t)row * p.HC + col);
        if constexpr (BY_SRC) ln.own_sl = p.sl[(int64_t)row * p.H + hd];
        else ln.own_rec = p.rec[(int64_t)row * p.H + hd];
    }
}

// One edge: nv = the neighbour's feature slice, nsl / nrec = the neighbour's scalars (zero when !ok).
// Runs with every lane of the wavefront active (the shuffle needs its partners).
// RECOMP (by destination only): the neighbour's sl is not gathered but recomputed from its feature slice --
// an fma chain from zero per lane, lanes added pairwise: the operations and the order of node_scores_kernel,
// hence the stored value bit for bit.
template <int VEC, bool BY_SRC, bool RECOMP>
__device__ __forceinline__ void lane_edge(Lane<VEC> &ln, const GatBwdParams &p, bool ok, const float *nv, float nsl,
                                          float4 nrec)
{
    float dot = 0.0f;
#pragma unroll
    for (int c = 0; c < VEC; ++c) dot = fmaf(ln.own[c], nv[c], dot);
    if constexpr (RECOMP) {
        nsl = 0.0f;
#pragma unroll
        for (int c = 0; c < VEC; ++c) nsl = fmaf(ln.as[c], nv[c], nsl);
    }
    // Over the head's lanes.  The usual widths get exchange patterns that are known when the kernel is compiled
    // (same pairwise order as the loop: neighbours first).
    if (p.lh == 2) {
        dot += __shfl_xor(dot, 1, 64);
        if constexpr (RECOMP) nsl += __shfl_xor(nsl, 1, 64);
    } else if (p.lh == 4) {
        dot += __shfl_xor(dot, 1, 64);
        dot += __shfl_xor(dot, 2, 64);
        if constexpr (RECOMP) { nsl += __shfl_xor(nsl, 1, 64); nsl += __shfl_xor(nsl, 2, 64); }
    } else if (p.lh_pow2) {
        for (int off = 1; off < p.lh; off <<= 1) {
            dot += __shfl_xor(dot, off, 64);
            if constexpr (RECOMP) nsl += __shfl_xor(nsl, off, 64);
        }
    } else {           // any lane count: every lane of the head adds the head's partial sums in lane order
        float tot = 0.0f;
        for (int t = 0; t < p.lh; ++t) tot += __shfl(dot, min(ln.head_first + t, 63), 64);
        dot = tot;
    }
    const float v = BY_SRC ? ln.own_sl + nrec.x : nsl + ln.own_rec.x;
    const float mx = BY_SRC ? nrec.y : ln.own_rec.y;
    const float inv = BY_SRC ? nrec.z : ln.own_rec.z;
    const float t = BY_SRC ? nrec.w : ln.own_rec.w;
    const bool pos = v > 0.0f;
    const float alpha = ok ? exp_hw((pos ? v : p.slope * v) - mx) * inv : 0.0f;
    ln.acc_s += alpha * (dot - t) * (pos ? 1.0f : p.slope);
    if constexpr (BY_SRC) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) ln.acc_v[c] = fmaf(alpha, nv[c], ln.acc_v[c]);
    }
}

template <int VEC, bool BY_SRC>
__device__ __forceinline__ void lane_write(const Lane<VEC> &ln, const GatBwdParams &p, int row, int col, int hd)
{
    if constexpr (BY_SRC) {
        // dh[i,hd,c] = sum of alpha G  +  dsl[i,hd] a_src[hd,c] + dsr[i,hd] a_dst[hd,c]: this row's dsl is the sum the
        // lane has just finished (the same in every lane of the head)
        float v[VEC];
        const float l = ln.acc_s, r = p.term_dsr[(int64_t)row * p.H + hd];
#pragma unroll
        for (int c = 0; c < VEC; ++c) v[c] = fmaf(l, p.a_src[col + c], fmaf(r, p.a_dst[col + c], ln.acc_v[c]));
        store_vec<VEC>(p.out_vec + (int64_t)row * p.HC + col, v);
    }
    if (col % p.ch == 0) p.out_s[(int64_t)row * p.H + hd] = ln.acc_s;
}

template <int LPR, int VEC, bool BY_SRC, bool RECOMP>
__device__ __forceinline__ void bwd_short_rows(const GatBwdParams &p, int block)
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

    for (int cb = 0; cb * p.pass_lanes * VEC < p.HC; ++cb) {
        const int col = (cb * p.pass_lanes + sl_) * VEC;
        const bool colok = have && sl_ < p.pass_lanes && col < p.HC;
        const int hd = colok ? col / p.ch : 0;
        Lane<VEC> ln;
        lane_init<VEC, BY_SRC, RECOMP>(ln, p, colok, row, col, hd);
        for (int base = 0; base < wmax; base += LPR) {
            int my_q = 0;
            if (base + sl_ < deg) my_q = p.colidx[start + base + sl_];
            const int cnt = min(LPR, wmax - base);
            for (int t0 = 0; t0 < cnt; t0 += U) {
                float nv[U][VEC], nsl[U];
                float4 nrec[U];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int t = t0 + u;
                    const int q = __shfl(my_q, t, LPR);
                    ok[u] = colok && (base + t < deg);
                    nsl[u] = 0.0f;
                    nrec[u] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int c = 0; c < VEC; ++c) nv[u][c] = 0.0f;
                    if (ok[u]) {
                        load_vec<VEC>(nv[u], p.nbr_vec + (int64_t)q * p.HC + col);
                        if constexpr (BY_SRC) nrec[u] = p.rec[(int64_t)q * p.H + hd];
                        else if constexpr (!RECOMP) nsl[u] = p.sl[(int64_t)q * p.H + hd];
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) lane_edge<VEC, BY_SRC, RECOMP>(ln, p, ok[u], nv[u], nsl[u], nrec[u]);
            }
        }
        if (colok) lane_write<VEC, BY_SRC>(ln, p, row, col, hd);
    }
}

template <int LPR, int VEC, bool BY_SRC, bool RECOMP>
__device__ __forceinline__ void bwd_long_pieces(const GatBwdParams &p, int block)
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

    for (int cb = 0; cb * p.pass_lanes * VEC < p.HC; ++cb) {
        const int col = (cb * p.pass_lanes + sl_) * VEC;
        const bool colok = sl_ < p.pass_lanes && col < p.HC;
        const int hd = colok ? col / p.ch : 0;
        Lane<VEC> ln;
        lane_init<VEC, BY_SRC, RECOMP>(ln, p, colok, row, col, hd);
        for (int base = start; base < end; base += 64) {
            const int n = min(64, end - base);
            int my_q = 0;
            if (lane < n) my_q = p.colidx[base + lane];
            for (int t0 = 0; t0 * NSG < n; t0 += U) {
                float nv[U][VEC], nsl[U];
                float4 nrec[U];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int pos = (t0 + u) * NSG + sg;
                    const int q = __shfl(my_q, pos, 64);
                    ok[u] = colok && pos < n;
                    nsl[u] = 0.0f;
                    nrec[u] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int c = 0; c < VEC; ++c) nv[u][c] = 0.0f;
                    if (ok[u]) {
                        load_vec<VEC>(nv[u], p.nbr_vec + (int64_t)q * p.HC + col);
                        if constexpr (BY_SRC) nrec[u] = p.rec[(int64_t)q * p.H + hd];
                        else if constexpr (!RECOMP) nsl[u] = p.sl[(int64_t)q * p.H + hd];
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) lane_edge<VEC, BY_SRC, RECOMP>(ln, p, ok[u], nv[u], nsl[u], nrec[u]);
            }
        }
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
            ln.acc_s += __shfl_xor(ln.acc_s, off, 64);
            if constexpr (BY_SRC) {
#pragma unroll
                for (int c = 0; c < VEC; ++c) ln.acc_v[c] += __shfl_xor(ln.acc_v[c], off, 64);
            }
        }
        if (sg == 0 && colok) {
            if (slot < 0) {
                lane_write<VEC, BY_SRC>(ln, p, row, col, hd);
            } else {
                const int64_t q = (int64_t)slot * p.HC + col;
                float sv[VEC];
#pragma unroll
                for (int c = 0; c < VEC; ++c) sv[c] = ln.acc_s;
                store_vec<VEC>(p.slot_s + q, sv);
                if constexpr (BY_SRC) store_vec<VEC>(p.slot_vec + q, ln.acc_v);
            }
        }
    }
}

template <int LPR, int VEC, bool BY_SRC, bool RECOMP>
__global__ __launch_bounds__(kThreads) void gat_backward_kernel(const GatBwdParams p)
{
    if ((int)blockIdx.x < p.item_blocks)
        bwd_long_pieces<LPR, VEC, BY_SRC, RECOMP>(p, blockIdx.x);
    else
        bwd_short_rows<LPR, VEC, BY_SRC, RECOMP>(p, blockIdx.x - p.item_blocks);
}

// Split rows: the pieces' partial sums are added in piece order.
template <int LPR, int VEC, bool BY_SRC>
__global__ __launch_bounds__(kThreads) void gat_backward_merge_kernel(const GatBwdParams p)
{
    const int64_t s = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / LPR;
    const int sl_ = threadIdx.x % LPR;
    if (s >= p.n_split) return;
    const int row = p.split_rows[s];
    const int slot0 = p.split_slot0[s];
    const int deg = p.rowptr[row + 1] - p.rowptr[row];
    const int pieces = (deg + p.chunk - 1) / p.chunk;
    for (int cb = 0; cb * p.pass_lanes * VEC < p.HC; ++cb) {
        const int col = (cb * p.pass_lanes + sl_) * VEC;
        if (sl_ >= p.pass_lanes || col >= p.HC) continue;
        Lane<VEC> ln;
        ln.acc_s = 0.0f;
#pragma unroll
        for (int c = 0; c < VEC; ++c) ln.acc_v[c] = 0.0f;
        for (int c = 0; c < pieces; ++c) {
            const int64_t q = (int64_t)(slot0 + c) * p.HC + col;
            ln.acc_s += p.slot_s[q];
            if constexpr (BY_SRC) {
                float v[VEC];
                load_vec<VEC>(v, p.slot_vec + q);
#pragma unroll
                for (int k = 0; k < VEC; ++k) ln.acc_v[k] += v[k];
            }
        }
        lane_write<VEC, BY_SRC>(ln, p, row, col, col / p.ch);
    }
}

// rec[i,hd] = (sr[i,hd], segment maximum, 1 / denominator (0 for an empty row), <G[i,hd,:], out[i,hd,:]>)
__global__ __launch_bounds__(kThreads) void node_records_kernel(const float *__restrict__ sr,
                                                                const float *__restrict__ stats,
                                                                const float *__restrict__ gout,
                                                                const float *__restrict__ out, int64_t N, int H,
                                                                int ch, int vec4, float4 *__restrict__ rec)
{
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= N * H) return;
    float t = 0.0f;
    if (vec4) {   // ch % 4 == 0 and both arrays 16-byte aligned
        const float4 *gp = reinterpret_cast<const float4 *>(gout + idx * ch), *op = reinterpret_cast<const float4 *>(out + idx * ch);
        for (int c = 0; c < ch / 4; ++c) {
            const float4 a = gp[c], b = op[c];
            t = fmaf(a.x, b.x, fmaf(a.y, b.y, fmaf(a.z, b.z, fmaf(a.w, b.w, t))));
        }
    } else {
        for (int c = 0; c < ch; ++c) t = fmaf(gout[idx * ch + c], out[idx * ch + c], t);
    }
    const float m = stats[2 * idx], d = stats[2 * idx + 1];
    rec[idx] = make_float4(sr[idx], d > 0.0f ? m : 0.0f, d > 0.0f ? 1.0f / d : 0.0f, t);
}

// partial_l[chunk][col] = sum over the chunk's rows of dsl[row,hd] h[row,col]; partial_r with dsr.
// A block's threads form (row slice, column) pairs: slice s takes rows s, s + slices, ... of the chunk
// and the slices are folded through LDS in slice order.
__global__ __launch_bounds__(kThreads) void attention_vector_partial_kernel(const float *__restrict__ h, int64_t N,
                                                                            int H, int ch,
                                                                            const float *__restrict__ dsl,
                                                                            const float *__restrict__ dsr,
                                                                            int64_t rows_per_chunk,
                                                                            float *__restrict__ partial_l,
                                                                            float *__restrict__ partial_r)
{
    __shared__ float fold_l[kThreads], fold_r[kThreads];
    const int HC = H * ch;
    const int cw = min(HC, kThreads), slices = kThreads / cw;
    const int rs = threadIdx.x / cw, c0 = threadIdx.x % cw;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_chunk, r1 = min(N, r0 + rows_per_chunk);
    for (int cbase = 0; cbase < HC; cbase += cw) {
        const int col = cbase + c0;
        float l[2] = {0.0f, 0.0f}, r[2] = {0.0f, 0.0f};   // two interleaved running sums each
        if (rs < slices && col < HC) {
            const int hd = col / ch;
            int64_t row = r0 + rs;
            for (; row + slices < r1; row += 2 * slices) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int64_t q = row + u * slices;
                    const float hv = h[q * HC + col];
                    l[u] = fmaf(dsl[q * H + hd], hv, l[u]);
                    r[u] = fmaf(dsr[q * H + hd], hv, r[u]);
                }
            }
            if (row < r1) {
                const float hv = h[row * HC + col];
                l[0] = fmaf(dsl[row * H + hd], hv, l[0]);
                r[0] = fmaf(dsr[row * H + hd], hv, r[0]);
            }
        }
        fold_l[threadIdx.x] = l[0] + l[1];
        fold_r[threadIdx.x] = r[0] + r[1];
        __syncthreads();
        if (rs == 0 && col < HC) {
            float sl_ = 0.0f, sr_ = 0.0f;
            for (int q = 0; q < slices; ++q) {
                sl_ += fold_l[q * cw + c0];
                sr_ += fold_r[q * cw + c0];
            }
            partial_l[(int64_t)blockIdx.x * HC + col] = sl_;
            partial_r[(int64_t)blockIdx.x * HC + col] = sr_;
        }
        __syncthreads();
    }
}

template <int LPR, int VEC, bool BY_SRC>
gnn_status launch_pass(const GatBwdParams &p, hipStream_t stream)
{
    constexpr int NSG = 64 / LPR;
    const int64_t blocks = p.item_blocks + gnn_div_up(p.n_small, kWavesPerBlock * NSG);
    if (blocks > 0) {
        // by destination, heads of at most 16 channels in 128-bit groups: sl[j] is recomputed from the gathered
        // slice in node_scores_kernel's tree order (wider heads are summed in another order there: gathered)
        constexpr bool kCanRecompute = !BY_SRC && VEC == 4;
        if (kCanRecompute && p.lh <= 4 && p.lh_pow2)
            hipLaunchKernelGGL((gat_backward_kernel<LPR, VEC, BY_SRC, kCanRecompute>), dim3((unsigned)blocks),
                               dim3(kThreads), 0, stream, p);
        else
            hipLaunchKernelGGL((gat_backward_kernel<LPR, VEC, BY_SRC, false>), dim3((unsigned)blocks), dim3(kThreads), 0,
                               stream, p);
        GNN_LAUNCH_CHECK();
    }
    if (p.n_split > 0) {
        const int64_t cblocks = gnn_div_up((int64_t)p.n_split * LPR, kThreads);
        hipLaunchKernelGGL((gat_backward_merge_kernel<LPR, VEC, BY_SRC>), dim3((unsigned)cblocks), dim3(kThreads), 0,
                           stream, p);
        GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
}

template <bool BY_SRC>
gnn_status run_pass(const gnn_graph *g, GatBwdParams p, bool vec4, hipStream_t s)
{
    p.rowptr = g->rowptr; p.colidx = g->colidx;
    p.small_rows = g->small_rows; p.item_row = g->item_row; p.item_start = g->item_start;
    p.item_slot = g->item_slot; p.split_rows = g->split_rows; p.split_slot0 = g->split_slot0;
    p.n_small = g->n_small; p.n_items = g->n_items; p.n_split = g->n_split; p.chunk = g->chunk;
    p.item_blocks = (int32_t)gnn_div_up(g->n_items, kWavesPerBlock);
    if (g->n_slots > 0) {
        float *scratch = nullptr;
        GNN_TRY(gnn_graph_scratch(g, 2 * (size_t)g->n_slots * p.HC, &scratch));
        p.slot_s = scratch;
        p.slot_vec = scratch + (size_t)g->n_slots * p.HC;
    }
    // lanes of a sub-group used per pass over a row (a sub-group is never narrower than a head)
    auto lanes = [&p](int lpr) { p.pass_lanes = p.lh_pow2 ? lpr : (lpr / p.lh) * p.lh; };
    if (vec4) {
        const int cols = p.HC / 4;
        if (cols <= 8) { lanes(8); return launch_pass<8, 4, BY_SRC>(p, s); }
        if (cols <= 16) { lanes(16); return launch_pass<16, 4, BY_SRC>(p, s); }
        if (cols <= 32) { lanes(32); return launch_pass<32, 4, BY_SRC>(p, s); }
        lanes(64);
        return launch_pass<64, 4, BY_SRC>(p, s);
    }
    if (p.HC <= 16) { lanes(16); return launch_pass<16, 1, BY_SRC>(p, s); }
    lanes(64);
    return launch_pass<64, 1, BY_SRC>(p, s);
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

struct Layout {
    size_t h, sl, sr, rec, dsl, dsr, dh, wt, part, total;
};

Layout layout(int64_t N, int f_in, int H, int ch)
{
    const int HC = H * ch;
    const size_t nhc = align256((size_t)N * HC * sizeof(float)), nh = align256((size_t)N * H * sizeof(float));
    const int chunks = gnn_row_chunk_count(N);
    Layout l{};
    l.h = 0;
    l.dh = l.h + nhc;
    l.sl = l.dh + nhc;
    l.sr = l.sl + nh;
    l.dsl = l.sr + nh;
    l.dsr = l.dsl + nh;
    l.rec = l.dsr + nh;
    l.wt = l.rec + align256((size_t)N * H * sizeof(float4));
    l.part = l.wt + align256((size_t)f_in * HC * sizeof(float));
    l.total = l.part + align256((size_t)chunks * std::max(f_in, 2) * HC * sizeof(float));
    return l;
}

bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

}  // namespace

extern "C" {

size_t gnn_gatconv_backward_workspace_bytes(int32_t num_nodes, int32_t f_in, int32_t heads, int32_t ch)
{
    if (num_nodes <= 0 || f_in <= 0 || heads <= 0 || ch <= 0) return 0;
    return layout(num_nodes, f_in, heads, ch).total;
}

gnn_status gnn_gatconv_backward(const gnn_graph *g, const gnn_graph *g_by_source, const float *d_x, int32_t f_in,
                                const float *d_w, const float *d_a_src, const float *d_a_dst, int32_t heads,
                                int32_t ch, float negative_slope, const float *d_out, const float *d_softmax_stats,
                                const float *d_grad_out, float *d_grad_x, float *d_grad_w, float *d_grad_a_src,
                                float *d_grad_a_dst, void *d_workspace, size_t workspace_bytes, void *stream)
{
    if (!g || !g_by_source || !d_x || !d_w || !d_a_src || !d_a_dst || !d_out || !d_softmax_stats || !d_grad_out ||
        !d_workspace)
        return GNN_ERR_NULL;
    if (f_in <= 0 || heads <= 0 || ch <= 0) return GNN_ERR_BAD_SIZE;
    if (g->bipartite) return GNN_ERR_UNSUPPORTED;   // one node set only
    if (g_by_source->num_nodes != g->num_nodes || g_by_source->num_edges != g->num_edges) return GNN_ERR_BAD_SIZE;
    const int64_t N = g->num_nodes;
    const int HC = heads * ch;
    const bool vec4 = (ch % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_grad_out) & 15u) == 0);
    const int lh = vec4 ? ch / 4 : ch;   // lanes that share a head
    // a head's lanes must lie in one wavefront (passes over a row start at head boundaries)
    if (lh > 64) return GNN_ERR_UNSUPPORTED;
    const Layout l = layout(N, f_in, heads, ch);
    if (workspace_bytes < l.total) return GNN_ERR_BAD_SIZE;
    if (reinterpret_cast<uintptr_t>(d_workspace) & 255u) return GNN_ERR_BAD_SIZE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(d_workspace);
    float *h = reinterpret_cast<float *>(ws + l.h), *dh = reinterpret_cast<float *>(ws + l.dh),
          *sl = reinterpret_cast<float *>(ws + l.sl), *sr = reinterpret_cast<float *>(ws + l.sr),
          *dsl = reinterpret_cast<float *>(ws + l.dsl), *dsr = reinterpret_cast<float *>(ws + l.dsr),
          *wt = reinterpret_cast<float *>(ws + l.wt), *part = reinterpret_cast<float *>(ws + l.part);
    float4 *rec = reinterpret_cast<float4 *>(ws + l.rec);

    // recomputed forward quantities and the per-node records
    GNN_TRY(gnn_dense_xw(d_x, N, f_in, d_w, HC, nullptr, h, stream));
    GNN_TRY(gnn_launch_node_scores(h, N, heads, ch, d_a_src, d_a_dst, sl, sr, s));
    hipLaunchKernelGGL(node_records_kernel, dim3((unsigned)gnn_div_up(N * heads, kThreads)), dim3(kThreads), 0, s, sr,
                       d_softmax_stats, d_grad_out, d_out, N, heads, ch,
                       (vec4 && (reinterpret_cast<uintptr_t>(d_out) & 15u) == 0) ? 1 : 0, rec);
    GNN_LAUNCH_CHECK();

    GatBwdParams p{};
    p.sl = sl; p.a_src = d_a_src; p.rec = rec;
    p.HC = HC; p.H = heads; p.ch = ch; p.lh = lh; p.lh_pow2 = is_pow2(lh) ? 1 : 0; p.slope = negative_slope;
    // by destination: dsr
    p.own_vec = d_grad_out; p.nbr_vec = h; p.out_vec = nullptr; p.out_s = dsr;
    GNN_TRY(run_pass<false>(g, p, vec4, s));
    // by source: dsl and the attention-weighted sum of G
    p.own_vec = h; p.nbr_vec = d_grad_out; p.out_vec = dh; p.out_s = dsl; p.a_dst = d_a_dst; p.term_dsr = dsr;
    GNN_TRY(run_pass<true>(g_by_source, p, vec4, s));

    const int chunks = gnn_row_chunk_count(N);
    const int64_t rows_per_chunk = gnn_div_up(N, chunks);
    if (d_grad_a_src || d_grad_a_dst) {
        float *part_l = part, *part_r = part + (size_t)chunks * HC;
        hipLaunchKernelGGL(attention_vector_partial_kernel, dim3((unsigned)chunks), dim3(kThreads), 0, s, h, N, heads,
                           ch, dsl, dsr, rows_per_chunk, part_l, part_r);
        GNN_LAUNCH_CHECK();
        if (d_grad_a_src) GNN_TRY(gnn_launch_sum_partials(part_l, chunks, HC, d_grad_a_src, s));
        if (d_grad_a_dst) GNN_TRY(gnn_launch_sum_partials(part_r, chunks, HC, d_grad_a_dst, s));
    }
    if (d_grad_w) GNN_TRY(gnn_launch_xty(d_x, dh, N, f_in, HC, part, d_grad_w, s));
    if (d_grad_x) {
        GNN_TRY(gnn_launch_xwt(dh, N, HC, d_w, f_in, nullptr, wt, d_grad_x, s));
    }
    return GNN_OK;
}

}  // extern "C"
