// propagate: gather of source-node feature rows along edges, per-edge message, segmented
// reduction onto destination nodes (paper section 3, "Message Passing": apply_edges followed
// by aggregate_neighbors, fused so that the [E x F] messages never exist in memory).
//
// Work decomposition over the by-destination CSR, chosen per row by in-degree when the graph
// is built:
//   * short rows  (in-degree <= small_max): one sub-group of LPR lanes per row, 64/LPR rows per
//     wavefront; the sub-group's lanes first fetch the row's neighbour ids (and weights) in one
//     coalesced load and hand them round by cross-lane shuffles, so all feature-row gathers of
//     a row are independent loads;
//   * long rows: pieces of at most `chunk` edges, one wavefront per piece; 64 neighbour ids are
//     fetched per step, the 64/LPR sub-groups take them round-robin and are combined with
//     xor-shuffles at the end;
//   * rows made of several pieces write per-piece partial rows to a scratch buffer and a second
//     kernel combines them in piece order, so results do not depend on scheduling (no atomics).
// A lane owns VEC consecutive features (VEC = 4: one 128-bit load per gathered row and lane).
#include "gnn_internal.h"

#include <algorithm>
#include <mutex>

// Scratch memory of gnn_propagate_noalloc: the partial rows of split rows for callers that must not touch the
// allocator at all.  A fixed array in the library's device image: every GPU the library runs on holds its own
// copy, at its own address, until the process ends.  Host code never uses the array's name as an address; it
// asks the runtime for the device address once per device (static_scratch_on_current_device) and passes that.
constexpr size_t kStaticScratchFloats = (size_t)4 << 20;   // 16 MiB
static __device__ __align__(256) float static_scratch[kStaticScratchFloats];

namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = kThreads / 64;

// Message kinds.  kMsgSubTarget is x_j - x_i (the row's own features are loaded once per row).
// The "routed" kinds (+4) are used by the backward pass of a max aggregation: the
// gathered row is the upstream gradient of the edge's destination and a feature only contributes
// if the recorded winner of that (destination, feature) is this very edge.
// kMsgMulSource is one weight per edge looked up by the edge's source node, w = e[j] (a diagonal scaling of x that
// is never written out); the row's self term is then scaled by e[row] as well.
enum { kMsgCopy = 0, kMsgMulScalar = 1, kMsgMulVector = 2, kMsgSubTarget = 3, kMsgRouted = 4, kMsgMulSource = 8 };
// Reductions.  min runs as max over negated messages, negated back at the end: negation is exact and
// turns "+0 above -0" into "-0 below +0".
enum { kRedSum = 0, kRedMax = 1, kRedProd = 2, kRedMin = 3 };
constexpr bool red_is_max(int red) { return red == kRedMax || red == kRedMin; }
constexpr bool msg_by_source(int msg) { return msg == kMsgMulSource; }
constexpr int msg_base(int msg) { return msg_by_source(msg) ? kMsgMulScalar : msg % kMsgRouted; }
constexpr bool msg_routed(int msg) { return msg >= kMsgRouted && msg < kMsgMulSource; }

struct PropParams {
    const int32_t *rowptr, *colidx, *perm;
    const float *x, *e;
    float *out, *scratch;
    const int32_t *small_rows, *item_row, *item_start, *item_slot, *split_rows, *split_slot0;
    int32_t n_small, n_items, n_split, chunk, F, e_coo, item_blocks;
    int32_t mean, relu, accumulate;
    float self_scale;
    const float *row_scale, *bias;
    const int32_t *winners;   // [rows of x][F] winning edge id per element (routed kinds only)
};

typedef float v4f __attribute__((ext_vector_type(4)));

template <int VEC>
struct Row {
    float v[VEC];
};

template <int VEC>
__device__ __forceinline__ void load_row(Row<VEC> &r, const float *__restrict__ p)
{
    if constexpr (VEC == 8) {
        const v4f t = reinterpret_cast<const v4f *>(p)[0], u = reinterpret_cast<const v4f *>(p)[1];
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
        r.v[4] = u.x; r.v[5] = u.y; r.v[6] = u.z; r.v[7] = u.w;
    } else if constexpr (VEC == 4) {
        const v4f t = *reinterpret_cast<const v4f *>(p);
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
    } else {
        r.v[0] = *p;
    }
}

// Streaming variants: data touched once (edge data, output rows) should not displace the
// feature rows that are gathered again and again from the caches.
template <int VEC>
__device__ __forceinline__ void load_row_stream(Row<VEC> &r, const float *__restrict__ p)
{
    if constexpr (VEC == 8) {
        const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
        const v4f u = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p) + 1);
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
        r.v[4] = u.x; r.v[5] = u.y; r.v[6] = u.z; r.v[7] = u.w;
    } else if constexpr (VEC == 4) {
        const v4f t = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(p));
        r.v[0] = t.x; r.v[1] = t.y; r.v[2] = t.z; r.v[3] = t.w;
    } else {
        r.v[0] = __builtin_nontemporal_load(p);
    }
}

template <int VEC>
__device__ __forceinline__ void store_row(float *__restrict__ p, const Row<VEC> &r)
{
    if constexpr (VEC == 8) {
        v4f t = {r.v[0], r.v[1], r.v[2], r.v[3]}, u = {r.v[4], r.v[5], r.v[6], r.v[7]};
        reinterpret_cast<v4f *>(p)[0] = t;
        reinterpret_cast<v4f *>(p)[1] = u;
    } else if constexpr (VEC == 4) {
        v4f t = {r.v[0], r.v[1], r.v[2], r.v[3]};
        *reinterpret_cast<v4f *>(p) = t;
    } else {
        *p = r.v[0];
    }
}

template <int VEC>
__device__ __forceinline__ void store_row_stream(float *__restrict__ p, const Row<VEC> &r)
{
    if constexpr (VEC == 8) {
        v4f t = {r.v[0], r.v[1], r.v[2], r.v[3]}, u = {r.v[4], r.v[5], r.v[6], r.v[7]};
        __builtin_nontemporal_store(t, reinterpret_cast<v4f *>(p));
        __builtin_nontemporal_store(u, reinterpret_cast<v4f *>(p) + 1);
    } else if constexpr (VEC == 4) {
        v4f t = {r.v[0], r.v[1], r.v[2], r.v[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<v4f *>(p));
    } else {
        __builtin_nontemporal_store(r.v[0], p);
    }
}

// Features x[elem ..].  XB = 1: the array holds bfloat16 (the upper half of a float), XB = 2: IEEE binary16,
// eight per 128-bit load; load_x only issues the load and keeps the four raw words (so that the loads of several
// edges stay in flight together), x_value widens value c exactly when it is used.  Sums and results stay in float.
template <int VEC, int XB>
__device__ __forceinline__ void load_x(Row<VEC> &r, const float *__restrict__ x, int64_t elem)
{
    if constexpr (XB == 0) {
        load_row<VEC>(r, x + elem);
    } else {
        static_assert(VEC == 8, "16-bit rows are read eight values at a time");
        const v4f w = *reinterpret_cast<const v4f *>(reinterpret_cast<const uint16_t *>(x) + elem);
        r.v[0] = w.x; r.v[1] = w.y; r.v[2] = w.z; r.v[3] = w.w;
    }
}

template <int VEC, int XB>
__device__ __forceinline__ float x_value(const Row<VEC> &r, int c)
{
    if constexpr (XB == 0) {
        return r.v[c];
    } else {
        const uint32_t w = __float_as_uint(r.v[c >> 1]);
        if constexpr (XB == 1) {
            return __uint_as_float((c & 1) ? (w & 0xffff0000u) : (w << 16));
        } else {
            // binary16 -> binary32 is exact: the hardware conversion (subnormal halves included: kernels are
            // built with 16-bit denormals enabled, and the parity tests cover them bit for bit)
            const uint16_t h = (uint16_t)((c & 1) ? (w >> 16) : (w & 0xffffu));
            return (float)__builtin_bit_cast(_Float16, h);
        }
    }
}

__device__ __forceinline__ int load_stream(const int32_t *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ float load_stream(const float *p) { return __builtin_nontemporal_load(p); }

// The larger of two finite floats; for the pair (-0, +0) the result is +0.
__device__ __forceinline__ float max_pz(float a, float b)
{
    // one v_max_f32: the hardware maximum orders -0 below +0 whichever operand comes first (checked on the
    // device: max(+0, -0) = max(-0, +0) = +0, max(-0, -0) = -0); inputs are finite.  Written as the instruction
    // itself: fmaxf() would first pass both operands through a NaN-quieting max of their own.
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

template <int VEC, int RED>
__device__ __forceinline__ void set_identity(Row<VEC> &r)
{
#pragma unroll
    for (int c = 0; c < VEC; ++c) r.v[c] = red_is_max(RED) ? -INFINITY : (RED == kRedProd ? 1.0f : 0.0f);
}

template <int VEC, int RED>
__device__ __forceinline__ void combine(Row<VEC> &acc, const Row<VEC> &m)
{
#pragma unroll
    for (int c = 0; c < VEC; ++c)
        acc.v[c] = red_is_max(RED) ? max_pz(acc.v[c], m.v[c]) : (RED == kRedProd ? acc.v[c] * m.v[c] : acc.v[c] + m.v[c]);
}

// Finishes one output row slice (VEC features starting at col) and stores it.
template <int VEC, int RED, int XB = 0, bool BYSRC = false>
__device__ __forceinline__ void finish_row(const PropParams &p, int row, int deg, int col, Row<VEC> acc)
{
    if constexpr (RED == kRedMin) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc.v[c] = -acc.v[c];
    }
    if (deg == 0) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc.v[c] = 0.0f;
    }
    if (p.mean && deg > 0) {
        const float d = (float)deg;
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc.v[c] = acc.v[c] / d;
    }
    if (p.self_scale != 0.0f) {
        Row<VEC> xs;
        load_x<VEC, XB>(xs, p.x, (int64_t)row * p.F + col);
        float ss = p.self_scale;
        if constexpr (BYSRC) ss *= p.e[row];
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc.v[c] = fmaf(ss, x_value<VEC, XB>(xs, c), acc.v[c]);
    }
    if (p.row_scale) {
        const float s = p.row_scale[row];
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc.v[c] *= s;
    }
    if (p.bias) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc.v[c] += p.bias[col + c];
    }
    if (p.relu) {
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc.v[c] = fmaxf(acc.v[c], 0.0f);
    }
    if (p.accumulate) {   // sum over the relations of a heterogeneous graph: add to what is there
        Row<VEC> old;
        load_row<VEC>(old, p.out + (int64_t)row * p.F + col);
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc.v[c] = old.v[c] + acc.v[c];
    }
    store_row_stream<VEC>(p.out + (int64_t)row * p.F + col, acc);
}

// Issues the loads of one gathered message: x[j, col..] and, for element-wise edge data, e[eid, col..].
// Nothing is computed here, so that the loads of several edges are in flight together; the
// message op is applied afterwards by apply_message.
template <int VEC, int MSG, int XB = 0>
__device__ __forceinline__ void fetch_message(const PropParams &p, bool ok, int j, int eid, int col, Row<VEC> &xv,
                                              Row<VEC> &ev, Row<VEC> &wv)
{
#pragma unroll
    for (int c = 0; c < VEC; ++c) { xv.v[c] = 0.0f; ev.v[c] = 0.0f; wv.v[c] = 0.0f; }
    if (ok) {
        load_x<VEC, XB>(xv, p.x, (int64_t)j * p.F + col);
        if constexpr (msg_base(MSG) == kMsgMulVector) load_row_stream<VEC>(ev, p.e + (int64_t)eid * p.F + col);
        if constexpr (msg_routed(MSG))   // winner ids travel as raw bits in a float row
            load_row<VEC>(wv, reinterpret_cast<const float *>(p.winners) + (int64_t)j * p.F + col);
    }
}

template <int VEC, int MSG, int RED, int XB = 0>
__device__ __forceinline__ void apply_message(Row<VEC> &acc, bool ok, const Row<VEC> &xv, float w, const Row<VEC> &ev,
                                              const Row<VEC> &wv, int eid, const Row<VEC> &xi)
{
#pragma unroll
    for (int c = 0; c < VEC; ++c) {
        float m = x_value<VEC, XB>(xv, c);
        if constexpr (msg_base(MSG) == kMsgMulScalar) m = w * m;
        if constexpr (msg_base(MSG) == kMsgMulVector) m = ev.v[c] * m;
        if constexpr (msg_base(MSG) == kMsgSubTarget) m = m - x_value<VEC, XB>(xi, c);
        if constexpr (msg_routed(MSG)) m = (__float_as_int(wv.v[c]) == eid) ? m : 0.0f;
        if constexpr (RED == kRedMin) m = -m;
        if constexpr (red_is_max(RED))
            acc.v[c] = ok ? max_pz(acc.v[c], m) : acc.v[c];
        else if constexpr (RED == kRedProd)
            acc.v[c] = ok ? acc.v[c] * m : acc.v[c];
        else if constexpr (msg_base(MSG) == kMsgSubTarget)
            acc.v[c] = acc.v[c] + (ok ? m : 0.0f);
        else
            acc.v[c] = acc.v[c] + m;   // masked-off edges carry x = 0
    }
}

template <int LPR, int VEC, int MSG, int RED, int XB>
__device__ __forceinline__ void short_rows(const PropParams &p, int block)
{
    constexpr int NSG = 64 / LPR;
    constexpr int U = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sl = lane % LPR, sg = lane / LPR;
    const int64_t sgid = ((int64_t)block * kWavesPerBlock + wave) * NSG + sg;
    const bool have = sgid < p.n_small;
    int row = 0, start = 0, deg = 0;
    if (have) {
        row = p.small_rows ? p.small_rows[sgid] : (int)sgid;   // no list: every row is short, the list is 0, 1, 2, ...
        start = p.rowptr[row];
        deg = p.rowptr[row + 1] - start;
    }
    int wmax = deg;   // loop bounds are kept uniform over the wavefront: shuffles run with all lanes active
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) wmax = max(wmax, __shfl_xor(wmax, off, 64));

    for (int cb = 0; cb * LPR * VEC < p.F; ++cb) {
        const int col = (cb * LPR + sl) * VEC;
        const bool colok = have && col < p.F;
        Row<VEC> acc, xi;
        set_identity<VEC, RED>(acc);
        set_identity<VEC, kRedSum>(xi);
        if constexpr (msg_base(MSG) == kMsgSubTarget)
            if (colok) load_x<VEC, XB>(xi, p.x, (int64_t)row * p.F + col);
        for (int base = 0; base < wmax; base += LPR) {
            int my_j = 0, my_eid = 0;
            float my_w = 0.0f;
            if (base + sl < deg) {
                const int q = start + base + sl;
                my_j = p.colidx ? load_stream(p.colidx + q) : q;   // no index array: row q itself
                if constexpr (msg_by_source(MSG)) {
                    my_w = p.e[my_j];
                } else if constexpr (MSG != kMsgCopy) {
                    my_eid = p.e_coo ? load_stream(p.perm + q) : q;
                    if constexpr (msg_base(MSG) == kMsgMulScalar) my_w = load_stream(p.e + my_eid);
                }
            }
            const int cnt = min(LPR, wmax - base);
            for (int t0 = 0; t0 < cnt; t0 += U) {
                Row<VEC> xv[U], ev[U], wv[U];
                int eid[U];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int t = t0 + u;
                    const int j = __shfl(my_j, t, LPR);
                    eid[u] = 0;
                    if constexpr (msg_base(MSG) == kMsgMulVector || msg_routed(MSG)) eid[u] = __shfl(my_eid, t, LPR);
                    ok[u] = colok && (base + t < deg);
                    fetch_message<VEC, MSG, XB>(p, ok[u], j, eid[u], col, xv[u], ev[u], wv[u]);
                }
                // the edges' weights are fetched from their lanes only after the loads have gone out (no register per
                // edge in flight); the barrier keeps the compiler from moving the shuffles up again
                if constexpr (msg_base(MSG) == kMsgMulScalar) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float w = 0.0f;
                    if constexpr (msg_base(MSG) == kMsgMulScalar) w = __shfl(my_w, t0 + u, LPR);
                    apply_message<VEC, MSG, RED, XB>(acc, ok[u], xv[u], w, ev[u], wv[u], eid[u], xi);
                }
            }
        }
        if (colok) finish_row<VEC, RED, XB, msg_by_source(MSG)>(p, row, deg, col, acc);
    }
}

template <int LPR, int VEC, int MSG, int RED, int XB>
__device__ __forceinline__ void long_row_pieces(const PropParams &p, int block)
{
    constexpr int NSG = 64 / LPR;
    constexpr int U = (LPR >= 4) ? 4 : LPR;   // gathers in flight per lane: more of them per wavefront did not pay (measured 2, 3, 4, 6, 8, 16)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sl = lane % LPR, sg = lane / LPR;
    const int it = block * kWavesPerBlock + wave;
    if (it >= p.n_items) return;   // whole wavefront leaves together
    const int row = p.item_row[it];
    const int start = p.item_start[it];
    const int slot = p.item_slot[it];
    const int row_start = p.rowptr[row], row_end = p.rowptr[row + 1];
    const int end = min(start + p.chunk, row_end);

    for (int cb = 0; cb * LPR * VEC < p.F; ++cb) {
        const int col = (cb * LPR + sl) * VEC;
        const bool colok = col < p.F;
        Row<VEC> acc, xi;
        set_identity<VEC, RED>(acc);
        set_identity<VEC, kRedSum>(xi);
        if constexpr (msg_base(MSG) == kMsgSubTarget)
            if (colok) load_x<VEC, XB>(xi, p.x, (int64_t)row * p.F + col);
        for (int base = start; base < end; base += 64) {
            const int n = min(64, end - base);
            int my_j = 0, my_eid = 0;
            float my_w = 0.0f;
            if (lane < n) {
                const int q = base + lane;
                my_j = p.colidx ? load_stream(p.colidx + q) : q;   // no index array: row q itself
                if constexpr (msg_by_source(MSG)) {
                    my_w = p.e[my_j];
                } else if constexpr (MSG != kMsgCopy) {
                    my_eid = p.e_coo ? load_stream(p.perm + q) : q;
                    if constexpr (msg_base(MSG) == kMsgMulScalar) my_w = load_stream(p.e + my_eid);
                }
            }
            // sub-group sg takes batch positions sg, sg + NSG, sg + 2*NSG, ...
            for (int t0 = 0; t0 * NSG < n; t0 += U) {
                Row<VEC> xv[U], ev[U], wv[U];
                int eid[U];
                bool ok[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int pos = (t0 + u) * NSG + sg;   // <= 63 because t0 + u < LPR
                    const int j = __shfl(my_j, pos, 64);
                    eid[u] = 0;
                    if constexpr (msg_base(MSG) == kMsgMulVector || msg_routed(MSG)) eid[u] = __shfl(my_eid, pos, 64);
                    ok[u] = colok && pos < n;
                    fetch_message<VEC, MSG, XB>(p, ok[u], j, eid[u], col, xv[u], ev[u], wv[u]);
                }
                if constexpr (msg_base(MSG) == kMsgMulScalar) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    float w = 0.0f;
                    if constexpr (msg_base(MSG) == kMsgMulScalar) w = __shfl(my_w, (t0 + u) * NSG + sg, 64);
                    apply_message<VEC, MSG, RED, XB>(acc, ok[u], xv[u], w, ev[u], wv[u], eid[u], xi);
                }
            }
        }
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
            Row<VEC> other;
#pragma unroll
            for (int c = 0; c < VEC; ++c) other.v[c] = __shfl_xor(acc.v[c], off, 64);
            combine<VEC, RED>(acc, other);
        }
        if (sg == 0 && colok) {
            if (slot < 0)
                finish_row<VEC, RED, XB, msg_by_source(MSG)>(p, row, row_end - row_start, col, acc);
            else
                store_row<VEC>(p.scratch + (int64_t)slot * p.F + col, acc);
        }
    }
}

// Blocks [0, item_blocks) take the long-row pieces (scheduled first: they are the heaviest),
// the remaining blocks take the short rows.
template <int LPR, int VEC, int MSG, int RED, int XB = 0>
__global__ __launch_bounds__(kThreads) void propagate_kernel(const PropParams p)
{
    if ((int)blockIdx.x < p.item_blocks)
        long_row_pieces<LPR, VEC, MSG, RED, XB>(p, blockIdx.x);
    else
        short_rows<LPR, VEC, MSG, RED, XB>(p, blockIdx.x - p.item_blocks);
}

// Combines the per-piece partial rows of split rows: one wavefront per split row, its sub-groups
// take the pieces round-robin (four loads in flight each) and are folded with xor-shuffles; the
// order of combination is a fixed function of the piece count.
template <int LPR, int VEC, int RED, int XB = 0, bool BYSRC = false>
__global__ __launch_bounds__(kThreads) void combine_pieces_kernel(const PropParams p)
{
    constexpr int NSG = 64 / LPR;
    constexpr int U = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sl = lane % LPR, sg = lane / LPR;
    const int s = blockIdx.x * kWavesPerBlock + wave;
    if (s >= p.n_split) return;   // whole wavefront leaves together
    const int row = p.split_rows[s];
    const int slot0 = p.split_slot0[s];
    const int deg = p.rowptr[row + 1] - p.rowptr[row];
    const int pieces = (deg + p.chunk - 1) / p.chunk;
    for (int cb = 0; cb * LPR * VEC < p.F; ++cb) {
        const int col = (cb * LPR + sl) * VEC;
        const bool colok = col < p.F;
        Row<VEC> acc;
        set_identity<VEC, RED>(acc);
        for (int c0 = sg; c0 < pieces; c0 += NSG * U) {
            Row<VEC> part[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = c0 + u * NSG;
                set_identity<VEC, RED>(part[u]);
                if (colok && c < pieces) load_row<VEC>(part[u], p.scratch + (int64_t)(slot0 + c) * p.F + col);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) combine<VEC, RED>(acc, part[u]);
        }
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
            Row<VEC> other;
#pragma unroll
            for (int c = 0; c < VEC; ++c) other.v[c] = __shfl_xor(acc.v[c], off, 64);
            combine<VEC, RED>(acc, other);
        }
        if (sg == 0 && colok) finish_row<VEC, RED, XB, BYSRC>(p, row, deg, col, acc);
    }
}

// apply_edges: one message row per edge, m[k,:] = msg(x[dst[k],:], x[src[k],:], e[k,:]), written in the caller's edge
// order or in CSR order.  One thread per (CSR position, VEC features).
template <int VEC, int MSG>
__global__ __launch_bounds__(kThreads) void apply_edges_kernel(const int32_t *__restrict__ colidx,
                                                               const int32_t *__restrict__ rowidx,
                                                               const int32_t *__restrict__ perm, int64_t E, int F,
                                                               const float *__restrict__ x,
                                                               const float *__restrict__ e, int e_coo, int m_coo,
                                                               float *__restrict__ m)
{
    const int cols = F / VEC;
    const int64_t total = E * cols;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total; idx += stride) {
        const int64_t q = idx / cols;
        const int col = (int)(idx - q * cols) * VEC;
        const int j = load_stream(colidx + q);
        const int64_t eid = (e_coo || m_coo) ? load_stream(perm + q) : q;
        Row<VEC> v;
        load_row<VEC>(v, x + (int64_t)j * F + col);
        if constexpr (MSG == kMsgMulScalar) {
            const float w = load_stream(e + (e_coo ? eid : q));
#pragma unroll
            for (int c = 0; c < VEC; ++c) v.v[c] = w * v.v[c];
        } else if constexpr (MSG == kMsgMulVector) {
            Row<VEC> ev;
            load_row_stream<VEC>(ev, e + (e_coo ? eid : q) * F + col);
#pragma unroll
            for (int c = 0; c < VEC; ++c) v.v[c] = ev.v[c] * v.v[c];
        } else if constexpr (MSG == kMsgSubTarget) {
            Row<VEC> xi;
            load_row<VEC>(xi, x + (int64_t)load_stream(rowidx + q) * F + col);
#pragma unroll
            for (int c = 0; c < VEC; ++c) v.v[c] = v.v[c] - xi.v[c];
        }
        store_row_stream<VEC>(m + (m_coo ? eid : q) * F + col, v);
    }
}

template <int LPR, int VEC, int MSG, int RED, int XB = 0>
gnn_status launch_typed(const PropParams &p, hipStream_t stream)
{
    constexpr int NSG = 64 / LPR;
    const int64_t small_blocks = gnn_div_up(p.n_small, kWavesPerBlock * NSG);
    const int64_t blocks = p.item_blocks + small_blocks;
    if (blocks > 0) {
        hipLaunchKernelGGL((propagate_kernel<LPR, VEC, MSG, RED, XB>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                           p);
        GNN_LAUNCH_CHECK();
    }
    if (p.n_split > 0) {
        const int64_t cblocks = gnn_div_up(p.n_split, kWavesPerBlock);
        hipLaunchKernelGGL((combine_pieces_kernel<LPR, VEC, RED, XB, msg_by_source(MSG)>), dim3((unsigned)cblocks), dim3(kThreads), 0, stream,
                           p);
        GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
}

template <int LPR, int VEC>
gnn_status launch_shape(const PropParams &p, int msg, int red, hipStream_t stream)
{
    switch (msg * 4 + red) {
    case kMsgCopy * 4 + kRedSum: return launch_typed<LPR, VEC, kMsgCopy, kRedSum>(p, stream);
    case kMsgCopy * 4 + kRedMax: return launch_typed<LPR, VEC, kMsgCopy, kRedMax>(p, stream);
    case kMsgCopy * 4 + kRedProd: return launch_typed<LPR, VEC, kMsgCopy, kRedProd>(p, stream);
    case kMsgCopy * 4 + kRedMin: return launch_typed<LPR, VEC, kMsgCopy, kRedMin>(p, stream);
    case kMsgMulScalar * 4 + kRedSum: return launch_typed<LPR, VEC, kMsgMulScalar, kRedSum>(p, stream);
    case kMsgMulScalar * 4 + kRedMax: return launch_typed<LPR, VEC, kMsgMulScalar, kRedMax>(p, stream);
    case kMsgMulScalar * 4 + kRedProd: return launch_typed<LPR, VEC, kMsgMulScalar, kRedProd>(p, stream);
    case kMsgMulScalar * 4 + kRedMin: return launch_typed<LPR, VEC, kMsgMulScalar, kRedMin>(p, stream);
    case kMsgMulVector * 4 + kRedSum: return launch_typed<LPR, VEC, kMsgMulVector, kRedSum>(p, stream);
    case kMsgMulVector * 4 + kRedMax: return launch_typed<LPR, VEC, kMsgMulVector, kRedMax>(p, stream);
    case kMsgMulVector * 4 + kRedProd: return launch_typed<LPR, VEC, kMsgMulVector, kRedProd>(p, stream);
    case kMsgMulVector * 4 + kRedMin: return launch_typed<LPR, VEC, kMsgMulVector, kRedMin>(p, stream);
    case kMsgSubTarget * 4 + kRedSum: return launch_typed<LPR, VEC, kMsgSubTarget, kRedSum>(p, stream);
    case kMsgSubTarget * 4 + kRedMax: return launch_typed<LPR, VEC, kMsgSubTarget, kRedMax>(p, stream);
    case kMsgSubTarget * 4 + kRedProd: return launch_typed<LPR, VEC, kMsgSubTarget, kRedProd>(p, stream);
    case kMsgSubTarget * 4 + kRedMin: return launch_typed<LPR, VEC, kMsgSubTarget, kRedMin>(p, stream);
    case kMsgMulSource * 4 + kRedSum: return launch_typed<LPR, VEC, kMsgMulSource, kRedSum>(p, stream);
    case (kMsgRouted + kMsgCopy) * 4 + kRedSum:
        return launch_typed<LPR, VEC, kMsgRouted + kMsgCopy, kRedSum>(p, stream);
    case (kMsgRouted + kMsgMulScalar) * 4 + kRedSum:
        return launch_typed<LPR, VEC, kMsgRouted + kMsgMulScalar, kRedSum>(p, stream);
    case (kMsgRouted + kMsgMulVector) * 4 + kRedSum:
        return launch_typed<LPR, VEC, kMsgRouted + kMsgMulVector, kRedSum>(p, stream);
    }
    return GNN_ERR_BAD_SIZE;
}

// Round-to-nearest-even conversion of finite floats to bfloat16 (the upper 16 bits of the float encoding).
__global__ __launch_bounds__(kThreads) void f32_to_bf16_kernel(const float *__restrict__ in, int64_t n,
                                                               uint16_t *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const uint32_t u = __float_as_uint(in[i]);
        out[i] = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
    }
}

// Round-to-nearest-even conversion of finite floats to IEEE binary16 with integer operations (and one float add in
// the default rounding mode for the subnormal range): |x| >= 65520 gives infinity, |x| < 2^-14 a subnormal code
// n = round(|x| * 2^24), else the float's 23-bit fraction is rounded to 10 bits and the exponent rebiased.
__global__ __launch_bounds__(kThreads) void f32_to_f16_kernel(const float *__restrict__ in, int64_t n,
                                                              uint16_t *__restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) {
        const uint32_t u = __float_as_uint(in[i]);
        const uint32_t sign = (u >> 16) & 0x8000u, a = u & 0x7fffffffu;
        uint32_t code;
        if (a >= 0x477ff000u) {            // 65520
            code = 0x7c00u;
        } else if (a < 0x38800000u) {      // below 2^-14: whole multiples of 2^-24
            // the fraction bits of |x| + 0.5 (for |x| < 2^-14 < 0.5 the sum lies in [0.5, 1), spacing 2^-24) are
            // |x| rounded to a multiple of 2^-24 by the float adder itself: round to nearest, ties to even
            // (fraction of 0.5 is zero, i.e. even)
            const float t = __uint_as_float(a) + 0.5f;
            code = __float_as_uint(t) - 0x3f000000u;   // = n, 0 .. 1024 (1024 = 0x0400 is the smallest normal)
        } else {
            const uint32_t r = a + 0xfffu + ((a >> 13) & 1u);
            code = (r >> 13) - (112u << 10);
        }
        out[i] = (uint16_t)(sign | code);
    }
}

// 16-bit feature storage (XB = 1 bfloat16, 2 binary16): copy_xj / one weight per edge, sum (mean) / max.
template <int LPR, int XB>
gnn_status launch_shape_16bit(const PropParams &p, int msg, int red, hipStream_t stream)
{
    switch (msg * 4 + red) {
    case kMsgCopy * 4 + kRedSum: return launch_typed<LPR, 8, kMsgCopy, kRedSum, XB>(p, stream);
    case kMsgCopy * 4 + kRedMax: return launch_typed<LPR, 8, kMsgCopy, kRedMax, XB>(p, stream);
    case kMsgMulScalar * 4 + kRedSum: return launch_typed<LPR, 8, kMsgMulScalar, kRedSum, XB>(p, stream);
    case kMsgMulScalar * 4 + kRedMax: return launch_typed<LPR, 8, kMsgMulScalar, kRedMax, XB>(p, stream);
    }
    return GNN_ERR_UNSUPPORTED;
}

template <int XB>
gnn_status launch_16bit(const PropParams &p, int cols, int msg, int red, hipStream_t stream)
{
    if (cols <= 8) return launch_shape_16bit<8, XB>(p, msg, red, stream);
    if (cols <= 16) return launch_shape_16bit<16, XB>(p, msg, red, stream);
    if (cols <= 32) return launch_shape_16bit<32, XB>(p, msg, red, stream);
    return launch_shape_16bit<64, XB>(p, msg, red, stream);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool valid_aggr(gnn_aggr a) { return a >= GNN_AGGR_SUM && a <= GNN_AGGR_PROD; }

int reduce_of(gnn_aggr a)
{
    switch (a) {
    case GNN_AGGR_MAX: return GNN_REDUCE_MAX;
    case GNN_AGGR_MIN: return GNN_REDUCE_MIN;
    case GNN_AGGR_PROD: return GNN_REDUCE_PROD;
    default: return GNN_REDUCE_SUM;
    }
}

constexpr int kMaxDevices = 64;
std::mutex g_static_scratch_mu;
float *g_static_scratch_ptr[kMaxDevices];   // device address of static_scratch, per device, once asked for

// The device address of this device's copy of static_scratch (looked up on the first call per device).
gnn_status static_scratch_on_current_device(float **out)
{
    int dev = 0;
    GNN_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return GNN_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_scratch_mu);
    if (!g_static_scratch_ptr[dev]) {
        void *p = nullptr;
        GNN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch)));
        if (!p) return GNN_ERR_DEVICE;
        g_static_scratch_ptr[dev] = static_cast<float *>(p);
    }
    *out = g_static_scratch_ptr[dev];
    return GNN_OK;
}

}  // namespace

gnn_status gnn_launch_propagate(const gnn_graph *g, const float *d_x, int32_t feat_dim, const float *d_e,
                                int32_t e_dim, gnn_edge_order e_order, gnn_msg_op msg, int reduce,
                                const gnn_epilogue &epi, float *d_out, hipStream_t stream, gnn_gather_index gather,
                                const int32_t *d_winners, int x_is_bf16, float *d_scratch, size_t scratch_floats)
{
    const int F = feat_dim;
    int kmsg = kMsgCopy;
    if (msg == GNN_MSG_E_MUL_XJ) kmsg = (e_dim == 1) ? kMsgMulScalar : kMsgMulVector;
    if (msg == GNN_MSG_XJ_SUB_XI) {
        if (gather != GNN_GATHER_SOURCE_NODE) return GNN_ERR_UNSUPPORTED;   // the row's own features are x[row]
        kmsg = kMsgSubTarget;
    }
    if (reduce < GNN_REDUCE_SUM || reduce > GNN_REDUCE_PROD) return GNN_ERR_BAD_SIZE;
    // x[row] (self term, x_j - x_i) only exists when sources and destinations are one node set
    if ((epi.self_scale != 0.0f || msg == GNN_MSG_XJ_SUB_XI) && g->bipartite)
        return GNN_ERR_UNSUPPORTED;
    if (d_winners) {
        if (reduce != GNN_REDUCE_SUM || e_order != GNN_EDGE_ORDER_COO || msg == GNN_MSG_XJ_SUB_XI)
            return GNN_ERR_UNSUPPORTED;   // edge ids are compared
        kmsg += kMsgRouted;
    }
    if (epi.source_scale) {   // a per-source weight is the one-weight-per-edge kernel with another index
        if (msg != GNN_MSG_COPY_XJ || reduce != GNN_REDUCE_SUM || gather != GNN_GATHER_SOURCE_NODE || d_winners ||
            x_is_bf16 || g->bipartite)
            return GNN_ERR_UNSUPPORTED;
        kmsg = kMsgMulSource;
    }
    const int red = reduce == GNN_REDUCE_SUM ? kRedSum
                    : reduce == GNN_REDUCE_PROD ? kRedProd : reduce == GNN_REDUCE_MIN ? kRedMin : kRedMax;

    // One weight per edge in the caller's order: with a route the weights are first moved to CSR order in two
    // streaming passes (into the route's staging buffer), which costs less than reading them through perm.
    if (kmsg == kMsgMulScalar && e_order == GNN_EDGE_ORDER_COO && g->route && g->num_edges > 0 && gnn_aligned16(d_e)) {
        GNN_TRY(gnn_route_coo_to_csr(g, d_e, g->route->staged, stream));
        d_e = g->route->staged;
        e_order = GNN_EDGE_ORDER_CSR;
    }

    PropParams p{};
    p.rowptr = g->rowptr; p.perm = g->perm;
    p.colidx = gather == GNN_GATHER_SOURCE_NODE ? g->colidx : (gather == GNN_GATHER_EDGE_COO ? g->perm : nullptr);
    p.x = d_x; p.e = epi.source_scale ? epi.source_scale : d_e; p.out = d_out;
    // when every row is short the ascending list of short rows is the identity: one dependent load less per row
    p.small_rows = (g->n_small == g->num_nodes) ? nullptr : g->small_rows; p.item_row = g->item_row; p.item_start = g->item_start;
    p.item_slot = g->item_slot; p.split_rows = g->split_rows; p.split_slot0 = g->split_slot0;
    p.n_small = g->n_small; p.n_items = g->n_items; p.n_split = g->n_split; p.chunk = g->chunk;
    p.F = F; p.e_coo = (e_order == GNN_EDGE_ORDER_COO) ? 1 : 0;
    p.item_blocks = (int32_t)gnn_div_up(g->n_items, kWavesPerBlock);
    p.mean = epi.mean; p.relu = epi.relu; p.accumulate = epi.accumulate; p.self_scale = epi.self_scale; p.row_scale = epi.row_scale; p.bias = epi.bias;
    p.winners = d_winners;

    if (d_scratch) {   // the caller's buffer for the partial rows instead of the graph's
        if ((size_t)g->n_slots * F > scratch_floats) return GNN_ERR_SCRATCH_LIMIT;
        p.scratch = d_scratch;
    } else {
        GNN_TRY(gnn_graph_scratch(g, (size_t)g->n_slots * F, &p.scratch));
    }

    if (x_is_bf16) {   // 1 = bfloat16, 2 = binary16
        if (F % 8 != 0 || !aligned16(d_x) || !aligned16(d_out) || d_winners) return GNN_ERR_UNSUPPORTED;
        if (x_is_bf16 == 1) return launch_16bit<1>(p, F / 8, kmsg, red, stream);
        return launch_16bit<2>(p, F / 8, kmsg, red, stream);
    }
    const bool vec4 = (F % 4 == 0) && aligned16(d_x) && aligned16(d_out) &&
                      (msg_base(kmsg) != kMsgMulVector || aligned16(d_e)) && aligned16(d_winners);
    if (vec4) {
        const int cols = F / 4;
        if (cols <= 4) return launch_shape<4, 4>(p, kmsg, red, stream);   // F <= 16: sixteen rows per wavefront
        if (cols <= 8) return launch_shape<8, 4>(p, kmsg, red, stream);
        if (cols <= 16) return launch_shape<16, 4>(p, kmsg, red, stream);
        if (cols <= 32) return launch_shape<32, 4>(p, kmsg, red, stream);
        return launch_shape<64, 4>(p, kmsg, red, stream);
    }
    if (F <= 16) return launch_shape<16, 1>(p, kmsg, red, stream);
    return launch_shape<64, 1>(p, kmsg, red, stream);
}

extern "C" {

static gnn_status check_propagate_arguments(const gnn_graph *g, const float *d_x, int32_t feat_dim, const float *d_e,
                                            int32_t e_dim, gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr,
                                            const float *d_out)
{
    if (!g || !d_x || !d_out) return GNN_ERR_NULL;
    if (feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (msg != GNN_MSG_COPY_XJ && msg != GNN_MSG_E_MUL_XJ && msg != GNN_MSG_XJ_SUB_XI) return GNN_ERR_BAD_SIZE;
    if (!valid_aggr(aggr)) return GNN_ERR_BAD_SIZE;
    if (msg == GNN_MSG_E_MUL_XJ) {
        if (e_dim != 1 && e_dim != feat_dim) return GNN_ERR_BAD_SIZE;
        if (e_order != GNN_EDGE_ORDER_COO && e_order != GNN_EDGE_ORDER_CSR) return GNN_ERR_BAD_SIZE;
        if (!d_e && g->num_edges > 0) return GNN_ERR_NULL;
    }
    return GNN_OK;
}

gnn_status gnn_propagate(const gnn_graph *g, const float *d_x, int32_t feat_dim, const float *d_e, int32_t e_dim,
                         gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr, float *d_out, void *stream)
{
    GNN_TRY(check_propagate_arguments(g, d_x, feat_dim, d_e, e_dim, e_order, msg, aggr, d_out));
    gnn_epilogue epi;
    epi.mean = (aggr == GNN_AGGR_MEAN);
    return gnn_launch_propagate(g, d_x, feat_dim, d_e, e_dim, e_order, msg, reduce_of(aggr), epi, d_out,
                                static_cast<hipStream_t>(stream));
}

gnn_status gnn_propagate_noalloc(const gnn_graph *g, const float *d_x, int32_t feat_dim, const float *d_e,
                                 int32_t e_dim, gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr, float *d_out,
                                 void *stream)
{
    GNN_TRY(check_propagate_arguments(g, d_x, feat_dim, d_e, e_dim, e_order, msg, aggr, d_out));
    if ((size_t)g->n_slots * (size_t)feat_dim > kStaticScratchFloats) return GNN_ERR_SCRATCH_LIMIT;
    float *d_scratch = nullptr;
    GNN_TRY(static_scratch_on_current_device(&d_scratch));
    gnn_epilogue epi;
    epi.mean = (aggr == GNN_AGGR_MEAN);
    // Nothing in the array has to start at zero: every partial row a launch reads was written by the same launch.
    return gnn_launch_propagate(g, d_x, feat_dim, d_e, e_dim, e_order, msg, reduce_of(aggr), epi, d_out,
                                static_cast<hipStream_t>(stream), GNN_GATHER_SOURCE_NODE, nullptr, 0, d_scratch,
                                kStaticScratchFloats);
}

gnn_status gnn_hetero_propagate(int32_t num_relations, const gnn_graph *const *graphs, const float *const *d_x,
                                const float *const *d_e, int32_t feat_dim, int32_t e_dim, gnn_edge_order e_order,
                                gnn_msg_op msg, gnn_aggr aggr, float *d_out, void *stream)
{
    if (num_relations <= 0 || feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (!graphs || !d_x || !d_out) return GNN_ERR_NULL;
    if (msg != GNN_MSG_COPY_XJ && msg != GNN_MSG_E_MUL_XJ) return msg == GNN_MSG_XJ_SUB_XI ? GNN_ERR_UNSUPPORTED
                                                                                           : GNN_ERR_BAD_SIZE;
    if (!valid_aggr(aggr)) return GNN_ERR_BAD_SIZE;
    if (msg == GNN_MSG_E_MUL_XJ) {
        if (!d_e) return GNN_ERR_NULL;
        if (e_dim != 1 && e_dim != feat_dim) return GNN_ERR_BAD_SIZE;
        if (e_order != GNN_EDGE_ORDER_COO && e_order != GNN_EDGE_ORDER_CSR) return GNN_ERR_BAD_SIZE;
    }
    for (int32_t r = 0; r < num_relations; ++r) {
        if (!graphs[r] || !d_x[r]) return GNN_ERR_NULL;
        if (graphs[r]->num_nodes != graphs[0]->num_nodes) return GNN_ERR_BAD_SIZE;
        if (msg == GNN_MSG_E_MUL_XJ && !d_e[r] && graphs[r]->num_edges > 0) return GNN_ERR_NULL;
    }
    for (int32_t r = 0; r < num_relations; ++r) {
        gnn_epilogue epi;
        epi.mean = (aggr == GNN_AGGR_MEAN);
        epi.accumulate = (r > 0);
        GNN_TRY(gnn_launch_propagate(graphs[r], d_x[r], feat_dim, d_e ? d_e[r] : nullptr, e_dim, e_order, msg,
                                     reduce_of(aggr), epi, d_out, static_cast<hipStream_t>(stream)));
    }
    return GNN_OK;
}

static gnn_status propagate_16bit(const gnn_graph *g, const uint16_t *d_x16, int storage, int32_t feat_dim,
                                  const float *d_e, gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr, float *d_out,
                                  void *stream)
{
    if (!g || !d_x16 || !d_out) return GNN_ERR_NULL;
    if (feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (!valid_aggr(aggr)) return GNN_ERR_BAD_SIZE;
    if (msg < GNN_MSG_COPY_XJ || msg > GNN_MSG_XI_DOT_XJ) return GNN_ERR_BAD_SIZE;
    if ((msg != GNN_MSG_COPY_XJ && msg != GNN_MSG_E_MUL_XJ) || aggr == GNN_AGGR_MIN || aggr == GNN_AGGR_PROD)
        return GNN_ERR_UNSUPPORTED;
    if (msg == GNN_MSG_E_MUL_XJ) {
        if (e_order != GNN_EDGE_ORDER_COO && e_order != GNN_EDGE_ORDER_CSR) return GNN_ERR_BAD_SIZE;
        if (!d_e && g->num_edges > 0) return GNN_ERR_NULL;
    }
    gnn_epilogue epi;
    epi.mean = (aggr == GNN_AGGR_MEAN);
    return gnn_launch_propagate(g, reinterpret_cast<const float *>(d_x16), feat_dim, d_e, 1, e_order, msg,
                                reduce_of(aggr), epi, d_out, static_cast<hipStream_t>(stream),
                                GNN_GATHER_SOURCE_NODE, nullptr, storage);
}

gnn_status gnn_propagate_bf16(const gnn_graph *g, const uint16_t *d_x_bf16, int32_t feat_dim, const float *d_e,
                              gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr, float *d_out, void *stream)
{
    return propagate_16bit(g, d_x_bf16, 1, feat_dim, d_e, e_order, msg, aggr, d_out, stream);
}

gnn_status gnn_propagate_f16(const gnn_graph *g, const uint16_t *d_x_f16, int32_t feat_dim, const float *d_e,
                             gnn_edge_order e_order, gnn_msg_op msg, gnn_aggr aggr, float *d_out, void *stream)
{
    return propagate_16bit(g, d_x_f16, 2, feat_dim, d_e, e_order, msg, aggr, d_out, stream);
}

gnn_status gnn_f32_to_bf16(const float *d_in, int64_t count, uint16_t *d_out, void *stream)
{
    if (count < 0) return GNN_ERR_BAD_SIZE;
    if (count == 0) return GNN_OK;
    if (!d_in || !d_out) return GNN_ERR_NULL;
    const int blocks = (int)std::min<int64_t>(gnn_div_up(count, kThreads), 256 * 64);
    hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream), d_in,
                       count, d_out);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_f32_to_f16(const float *d_in, int64_t count, uint16_t *d_out, void *stream)
{
    if (count < 0) return GNN_ERR_BAD_SIZE;
    if (count == 0) return GNN_OK;
    if (!d_in || !d_out) return GNN_ERR_NULL;
    const int blocks = (int)std::min<int64_t>(gnn_div_up(count, kThreads), 256 * 64);
    hipLaunchKernelGGL(f32_to_f16_kernel, dim3(blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream), d_in,
                       count, d_out);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_apply_edges(const gnn_graph *g, const float *d_x, int32_t feat_dim, const float *d_e, int32_t e_dim,
                           gnn_edge_order e_order, gnn_msg_op msg, float *d_m, gnn_edge_order m_order, void *stream)
{
    if (!g) return GNN_ERR_NULL;
    if (feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (msg < GNN_MSG_COPY_XJ || msg > GNN_MSG_XI_DOT_XJ) return GNN_ERR_BAD_SIZE;
    if (m_order != GNN_EDGE_ORDER_COO && m_order != GNN_EDGE_ORDER_CSR) return GNN_ERR_BAD_SIZE;
    if (msg == GNN_MSG_E_MUL_XJ) {
        if (e_dim != 1 && e_dim != feat_dim) return GNN_ERR_BAD_SIZE;
        if (e_order != GNN_EDGE_ORDER_COO && e_order != GNN_EDGE_ORDER_CSR) return GNN_ERR_BAD_SIZE;
    }
    if (g->num_edges == 0) return GNN_OK;
    if (!d_x || !d_m || (msg == GNN_MSG_E_MUL_XJ && !d_e)) return GNN_ERR_NULL;
    if ((msg == GNN_MSG_XI_DOT_XJ || msg == GNN_MSG_XJ_SUB_XI) && g->bipartite)
        return GNN_ERR_UNSUPPORTED;
    if (msg == GNN_MSG_XI_DOT_XJ) return gnn_launch_edge_dot(g, d_x, d_x, feat_dim, d_m, m_order, stream);
    int kmsg = kMsgCopy;
    if (msg == GNN_MSG_E_MUL_XJ) kmsg = (e_dim == 1) ? kMsgMulScalar : kMsgMulVector;
    if (msg == GNN_MSG_XJ_SUB_XI) kmsg = kMsgSubTarget;
    const int F = feat_dim;
    const bool vec4 = (F % 4 == 0) && aligned16(d_x) && aligned16(d_m) && (kmsg != kMsgMulVector || aligned16(d_e));
    const int64_t total = g->num_edges * (vec4 ? F / 4 : F);
    const dim3 grid((unsigned)std::min<int64_t>(gnn_div_up(total, kThreads), 256 * 128)), block(kThreads);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (kmsg == kMsgMulScalar && e_order == GNN_EDGE_ORDER_COO && g->route && gnn_aligned16(d_e)) {
        // one weight per edge in the caller's order: moved to CSR order in two streaming passes first
        GNN_TRY(gnn_route_coo_to_csr(g, d_e, g->route->staged, s));
        d_e = g->route->staged;
        e_order = GNN_EDGE_ORDER_CSR;
    }
    const int e_coo = (e_order == GNN_EDGE_ORDER_COO), m_coo = (m_order == GNN_EDGE_ORDER_COO);
#define GNN_APPLY(VEC, MSG)                                                                                      \
    hipLaunchKernelGGL((apply_edges_kernel<VEC, MSG>), grid, block, 0, s, g->colidx, g->rowidx, g->perm, g->num_edges, \
                       F, d_x, d_e, e_coo, m_coo, d_m)
    if (vec4) {
        if (kmsg == kMsgCopy) GNN_APPLY(4, kMsgCopy);
        else if (kmsg == kMsgMulScalar) GNN_APPLY(4, kMsgMulScalar);
        else if (kmsg == kMsgMulVector) GNN_APPLY(4, kMsgMulVector);
        else GNN_APPLY(4, kMsgSubTarget);
    } else {
        if (kmsg == kMsgCopy) GNN_APPLY(1, kMsgCopy);
        else if (kmsg == kMsgMulScalar) GNN_APPLY(1, kMsgMulScalar);
        else if (kmsg == kMsgMulVector) GNN_APPLY(1, kMsgMulVector);
        else GNN_APPLY(1, kMsgSubTarget);
    }
#undef GNN_APPLY
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_aggregate_neighbors(const gnn_graph *g, const float *d_m, int32_t feat_dim, gnn_edge_order m_order,
                                   gnn_aggr aggr, float *d_out, void *stream)
{
    if (!g || !d_out) return GNN_ERR_NULL;
    if (feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (!valid_aggr(aggr)) return GNN_ERR_BAD_SIZE;
    if (m_order != GNN_EDGE_ORDER_COO && m_order != GNN_EDGE_ORDER_CSR) return GNN_ERR_BAD_SIZE;
    if (!d_m && g->num_edges > 0) return GNN_ERR_NULL;
    gnn_epilogue epi;
    epi.mean = (aggr == GNN_AGGR_MEAN);
    return gnn_launch_propagate(g, d_m, feat_dim, nullptr, 1, GNN_EDGE_ORDER_CSR, GNN_MSG_COPY_XJ,
                                reduce_of(aggr), epi, d_out, static_cast<hipStream_t>(stream),
                                m_order == GNN_EDGE_ORDER_COO ? GNN_GATHER_EDGE_COO : GNN_GATHER_EDGE_CSR);
}

gnn_status gnn_gin_update(const gnn_graph *g, const float *d_x, int32_t feat_dim, float eps, float *d_out,
                          void *stream)
{
    if (!g || !d_x || !d_out) return GNN_ERR_NULL;
    if (feat_dim <= 0) return GNN_ERR_BAD_SIZE;
    gnn_epilogue epi;
    epi.self_scale = 1.0f + eps;
    return gnn_launch_propagate(g, d_x, feat_dim, nullptr, 1, GNN_EDGE_ORDER_CSR, GNN_MSG_COPY_XJ, 0, epi, d_out,
                                static_cast<hipStream_t>(stream));
}

}  // extern "C"
