// One float per edge between the caller's edge order and CSR order (the edge features e of the paper's section 3,
// "Message Passing", which are stored per edge of the COO list while the kernels walk the edges by destination).
//
// out[p] = e[perm[p]] read directly is 20 M random 4-byte reads for 20 M edges, and every one of them costs a whole
// 128-byte line.  perm is fixed per graph, so the permutation is split once into pieces that only move data inside
// LDS-sized ranges or in contiguous runs:
//   edge ids are cut into tiles and CSR positions into buckets of kRouteTile entries each;
//   the intermediate array `mid` is ordered by (bucket, edge id): bucket b occupies mid[b T, (b+1) T), like the
//   positions it feeds, and inside it the items are in increasing edge id -- so what one tile sends to one bucket
//   is one contiguous run of mid;
//   tile pass   (a block per tile):   the tile of e is read into LDS, item k of the tile in (bucket, edge id) order
//                                     is lds[tile_src[k]] and goes to mid[tile_dst[k]]: consecutive k, consecutive
//                                     addresses inside a run;
//   bucket pass (a block per bucket): the bucket of mid is read into LDS, out[p] = lds[bucket_idx[p]].
// The way back runs the same two passes mirrored (LDS scatter instead of LDS gather, run-wise global gather instead
// of scatter) with the same three index arrays.  Both directions move 24 bytes per edge in streams.
#include <algorithm>

#include "gnn_internal.h"

namespace {

constexpr int kRouteTile = 16384;     // edge ids per tile = CSR positions per bucket (64 KB of floats in LDS)
constexpr int kRouteThreads = 1024;
constexpr int kDies = 8;

typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned short v4u16 __attribute__((ext_vector_type(4)));

// Blocks are dealt round-robin to the eight dies; a die takes a contiguous range of tiles so that the runs two
// neighbouring tiles send to one bucket (neighbours in memory) meet in one L2.
__device__ inline int tile_of_block(int block, int tiles)
{
    const int per_die = (tiles + kDies - 1) / kDies;
    return (block % kDies) * per_die + block / kDies;
}

__device__ inline int entries_from(int64_t base, int64_t E)
{
    const int64_t left = E - base;
    return (int)(left < kRouteTile ? left : kRouteTile);
}

// ---------------------------------------------------------------- building the route (once per graph)
// Sorts the (key, local index) pairs of one range of kRouteTile keys in LDS (bitonic network; keys are distinct) and
// writes what the two sides of the route need:
//   BY_BUCKET: keys = perm of the bucket's positions (edge ids).  Rank k of local position l:
//              slot_of_edge[edge id] = base + k,  bucket_idx[base + l] = k.
//   by tile:   keys = slot_of_edge of the tile's edge ids.  Rank k of local edge l:
//              tile_dst[base + k] = slot,  tile_src[base + k] = l.
template <bool BY_BUCKET>
__global__ __launch_bounds__(kRouteThreads) void route_sort_kernel(const int32_t *__restrict__ keys, int64_t E,
                                                                   int32_t *__restrict__ out32,
                                                                   uint16_t *__restrict__ out16)
{
    extern __shared__ unsigned long long items[];
    const int64_t base = (int64_t)blockIdx.x * kRouteTile;
    const int n = entries_from(base, E);
    int m = 2;
    while (m < n) m <<= 1;
    for (int l = threadIdx.x; l < m; l += kRouteThreads)
        items[l] = l < n ? (((unsigned long long)(uint32_t)keys[base + l]) << 16) | (unsigned long long)l : ~0ull;
    __syncthreads();
    for (int size = 2; size <= m; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int pr = threadIdx.x; pr < (m >> 1); pr += kRouteThreads) {
                const int lo = 2 * pr - (pr & (stride - 1));
                const int hi = lo + stride;
                const unsigned long long a = items[lo], b = items[hi];
                const bool ascending = (lo & size) == 0;
                if ((a > b) == ascending) {
                    items[lo] = b;
                    items[hi] = a;
                }
            }
            __syncthreads();
        }
    }
    for (int k = threadIdx.x; k < n; k += kRouteThreads) {
        const unsigned long long it = items[k];
        const int64_t key = (int64_t)(it >> 16);
        const int l = (int)(it & 0xffffu);
        if constexpr (BY_BUCKET) {
            if (key < E) out32[key] = (int32_t)(base + k);
            out16[base + l] = (uint16_t)k;
        } else {
            out32[base + k] = (int32_t)key;
            out16[base + k] = (uint16_t)l;
        }
    }
}

// ---------------------------------------------------------------- the passes
// Index values are clamped to their range before use: with a correct route the clamps never act.

// tile pass, towards CSR order:  mid[tile_dst[k]] = e_tile[tile_src[k]]
__global__ __launch_bounds__(kRouteThreads) void route_tile_forward_kernel(const float *__restrict__ e,
                                                                           const uint16_t *__restrict__ tile_src,
                                                                           const int32_t *__restrict__ tile_dst,
                                                                           float *__restrict__ mid, int64_t E, int tiles)
{
    extern __shared__ float lds[];
    const int tile = tile_of_block(blockIdx.x, tiles);
    if (tile >= tiles) return;
    const int64_t base = (int64_t)tile * kRouteTile;
    const int n = entries_from(base, E);
    for (int k = threadIdx.x * 4; k < n; k += kRouteThreads * 4) {
        if (k + 3 < n) {
            *(v4f *)(lds + k) = __builtin_nontemporal_load((const v4f *)(e + base + k));
        } else {
            for (int c = 0; k + c < n; ++c) lds[k + c] = e[base + k + c];
        }
    }
    __syncthreads();
    const uint32_t last = (uint32_t)(n - 1);
    const int64_t last_slot = E - 1;
#pragma unroll 16
    for (int k = threadIdx.x; k < n; k += kRouteThreads) {
        const uint32_t src = __builtin_nontemporal_load(tile_src + base + k);
        int64_t dst = __builtin_nontemporal_load(tile_dst + base + k);
        dst = dst < 0 ? 0 : (dst > last_slot ? last_slot : dst);
        mid[dst] = lds[src < last ? src : last];
    }
}

// tile pass, towards the caller's order:  e_tile[tile_src[k]] = mid[tile_dst[k]]
__global__ __launch_bounds__(kRouteThreads) void route_tile_reverse_kernel(const float *__restrict__ mid,
                                                                           const uint16_t *__restrict__ tile_src,
                                                                           const int32_t *__restrict__ tile_dst,
                                                                           float *__restrict__ e, int64_t E, int tiles)
{
    extern __shared__ float lds[];
    const int tile = tile_of_block(blockIdx.x, tiles);
    if (tile >= tiles) return;
    const int64_t base = (int64_t)tile * kRouteTile;
    const int n = entries_from(base, E);
    const uint32_t last = (uint32_t)(n - 1);
    const int64_t last_slot = E - 1;
#pragma unroll 16
    for (int k = threadIdx.x; k < n; k += kRouteThreads) {
        const uint32_t dst = __builtin_nontemporal_load(tile_src + base + k);
        int64_t src = __builtin_nontemporal_load(tile_dst + base + k);
        src = src < 0 ? 0 : (src > last_slot ? last_slot : src);
        lds[dst < last ? dst : last] = mid[src];
    }
    __syncthreads();
    for (int k = threadIdx.x * 4; k < n; k += kRouteThreads * 4) {
        if (k + 3 < n) {
            __builtin_nontemporal_store(*(v4f *)(lds + k), (v4f *)(e + base + k));
        } else {
            for (int c = 0; k + c < n; ++c) e[base + k + c] = lds[k + c];
        }
    }
}

// bucket pass.  GATHER: out[base + k] = in[base + idx[base + k]]  (towards CSR order: in = mid);
//               else:   out[base + idx[base + k]] = in[base + k]  (towards the caller's order: out = mid).
template <bool GATHER>
__global__ __launch_bounds__(kRouteThreads) void route_bucket_kernel(const float *__restrict__ in,
                                                                     const uint16_t *__restrict__ idx,
                                                                     float *__restrict__ out, int64_t E)
{
    extern __shared__ float lds[];
    const int64_t base = (int64_t)blockIdx.x * kRouteTile;
    const int n = entries_from(base, E);
    const uint32_t last = (uint32_t)(n - 1);
    auto clamp = [last](uint32_t r) { return r < last ? r : last; };
    for (int k = threadIdx.x * 4; k < n; k += kRouteThreads * 4) {
        if (k + 3 < n) {
            const v4f v = __builtin_nontemporal_load((const v4f *)(in + base + k));
            if constexpr (GATHER) {
                *(v4f *)(lds + k) = v;
            } else {
                const v4u16 r = __builtin_nontemporal_load((const v4u16 *)(idx + base + k));
                lds[clamp(r.x)] = v.x;
                lds[clamp(r.y)] = v.y;
                lds[clamp(r.z)] = v.z;
                lds[clamp(r.w)] = v.w;
            }
        } else {
            for (int c = 0; k + c < n; ++c) {
                if constexpr (GATHER) lds[k + c] = in[base + k + c];
                else lds[clamp(idx[base + k + c])] = in[base + k + c];
            }
        }
    }
    __syncthreads();
    for (int k = threadIdx.x * 4; k < n; k += kRouteThreads * 4) {
        if (k + 3 < n) {
            v4f v;
            if constexpr (GATHER) {
                const v4u16 r = __builtin_nontemporal_load((const v4u16 *)(idx + base + k));
                v.x = lds[clamp(r.x)];
                v.y = lds[clamp(r.y)];
                v.z = lds[clamp(r.z)];
                v.w = lds[clamp(r.w)];
            } else {
                v = *(v4f *)(lds + k);
            }
            __builtin_nontemporal_store(v, (v4f *)(out + base + k));
        } else {
            for (int c = 0; k + c < n; ++c) {
                if constexpr (GATHER) out[base + k + c] = lds[clamp(idx[base + k + c])];
                else out[base + k + c] = lds[k + c];
            }
        }
    }
}

// the direct way back for any record width:  e_coo[perm[p], :] = e_csr[p, :]
__global__ __launch_bounds__(256) void unpermute_rows_kernel(const int32_t *__restrict__ perm, int64_t E,
                                                             const float *__restrict__ e_csr, int32_t e_dim,
                                                             float *__restrict__ e_coo)
{
    const int64_t total = E * e_dim;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x; q < total; q += stride) {
        const int64_t p = q / e_dim;
        const int32_t c = (int32_t)(q - p * e_dim);
        e_coo[(int64_t)perm[p] * e_dim + c] = e_csr[q];
    }
}

constexpr size_t kSortLdsBytes = (size_t)kRouteTile * sizeof(unsigned long long);   // 128 KB
constexpr size_t kPassLdsBytes = (size_t)kRouteTile * sizeof(float);                // 64 KB

gnn_status allow_lds(const void *kernel, size_t bytes)
{
    GNN_HIP(hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    return GNN_OK;
}

size_t align256(size_t bytes) { return (bytes + 255) & ~(size_t)255; }

}  // namespace

void gnn_route_free(gnn_graph *g)
{
    if (!g || !g->route) return;
    if (g->route->alloc) (void)hipFree(g->route->alloc);
    delete g->route;
    g->route = nullptr;
}

gnn_status gnn_route_coo_to_csr(const gnn_graph *g, const float *d_in, float *d_out, hipStream_t s)
{
    const gnn_edge_route *r = g->route;
    const int64_t E = g->num_edges;
    if (!r) return GNN_ERR_UNSUPPORTED;
    if (E == 0) return GNN_OK;
    const int tiles = (int)gnn_div_up(E, kRouteTile);
    const int tile_blocks = (int)gnn_div_up(tiles, kDies) * kDies;
    hipLaunchKernelGGL(route_tile_forward_kernel, dim3(tile_blocks), dim3(kRouteThreads), kPassLdsBytes, s, d_in,
                       r->tile_src, r->tile_dst, r->mid, E, tiles);
    GNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(route_bucket_kernel<true>, dim3(tiles), dim3(kRouteThreads), kPassLdsBytes, s, r->mid,
                       r->bucket_idx, d_out, E);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status gnn_route_csr_to_coo(const gnn_graph *g, const float *d_in, float *d_out, hipStream_t s)
{
    const gnn_edge_route *r = g->route;
    const int64_t E = g->num_edges;
    if (!r) return GNN_ERR_UNSUPPORTED;
    if (E == 0) return GNN_OK;
    const int tiles = (int)gnn_div_up(E, kRouteTile);
    const int tile_blocks = (int)gnn_div_up(tiles, kDies) * kDies;
    hipLaunchKernelGGL(route_bucket_kernel<false>, dim3(tiles), dim3(kRouteThreads), kPassLdsBytes, s, d_in,
                       r->bucket_idx, r->mid, E);
    GNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(route_tile_reverse_kernel, dim3(tile_blocks), dim3(kRouteThreads), kPassLdsBytes, s, r->mid,
                       r->tile_src, r->tile_dst, d_out, E, tiles);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

extern "C" {

gnn_status gnn_graph_build_edge_route(gnn_graph *g, void *stream)
{
    if (!g) return GNN_ERR_NULL;
    if (g->route) return GNN_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t E = g->num_edges;
    gnn_edge_route *r = new gnn_edge_route;
    if (E == 0) {
        g->route = r;
        return GNN_OK;
    }
    // tile_dst [E] int32 | mid [E] float | staged [E] float | tile_src [E] u16 | bucket_idx [E] u16
    const size_t words = align256((size_t)E * 4), halves = align256((size_t)E * 2);
    void *p = nullptr;
    if (hipMalloc(&p, 3 * words + 2 * halves) != hipSuccess) {
        (void)hipGetLastError();
        delete r;
        return GNN_ERR_ALLOC;
    }
    char *c = static_cast<char *>(p);
    r->alloc = p;
    r->tile_dst = reinterpret_cast<int32_t *>(c);
    r->mid = reinterpret_cast<float *>(c + words);
    r->staged = reinterpret_cast<float *>(c + 2 * words);
    r->tile_src = reinterpret_cast<uint16_t *>(c + 3 * words);
    r->bucket_idx = reinterpret_cast<uint16_t *>(c + 3 * words + halves);

    gnn_status st = allow_lds((const void *)route_sort_kernel<true>, kSortLdsBytes);
    if (st == GNN_OK) st = allow_lds((const void *)route_sort_kernel<false>, kSortLdsBytes);
    if (st == GNN_OK) st = allow_lds((const void *)route_tile_forward_kernel, kPassLdsBytes);
    if (st == GNN_OK) st = allow_lds((const void *)route_tile_reverse_kernel, kPassLdsBytes);
    if (st == GNN_OK) st = allow_lds((const void *)route_bucket_kernel<true>, kPassLdsBytes);
    if (st == GNN_OK) st = allow_lds((const void *)route_bucket_kernel<false>, kPassLdsBytes);
    if (st == GNN_OK) {
        const int tiles = (int)gnn_div_up(E, kRouteTile);
        int m = 2;
        while (m < std::min<int64_t>(E, kRouteTile)) m <<= 1;
        const size_t lds = (size_t)m * sizeof(unsigned long long);
        // the slot of every edge id (a temporary: it lives in `staged` until the second kernel has read it)
        int32_t *slot_of_edge = reinterpret_cast<int32_t *>(r->staged);
        hipLaunchKernelGGL(route_sort_kernel<true>, dim3(tiles), dim3(kRouteThreads), lds, s, g->perm, E, slot_of_edge,
                           r->bucket_idx);
        if (hipGetLastError() != hipSuccess) st = GNN_ERR_DEVICE;
        if (st == GNN_OK) {
            hipLaunchKernelGGL(route_sort_kernel<false>, dim3(tiles), dim3(kRouteThreads), lds, s, slot_of_edge, E,
                               r->tile_dst, r->tile_src);
            if (hipGetLastError() != hipSuccess) st = GNN_ERR_DEVICE;
        }
        if (st == GNN_OK && hipStreamSynchronize(s) != hipSuccess) {
            (void)hipGetLastError();
            st = GNN_ERR_DEVICE;
        }
    }
    if (st != GNN_OK) {
        (void)hipFree(p);
        delete r;
        return st;
    }
    g->route = r;
    return GNN_OK;
}

gnn_status gnn_edge_data_to_coo(const gnn_graph *g, const float *d_e_csr, int32_t e_dim, float *d_e, void *stream)
{
    if (!g) return GNN_ERR_NULL;
    if (e_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (g->num_edges == 0) return GNN_OK;
    if (!d_e || !d_e_csr) return GNN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (e_dim == 1 && g->route && gnn_aligned16(d_e) && gnn_aligned16(d_e_csr)) return gnn_route_csr_to_coo(g, d_e_csr, d_e, s);
    const int64_t total = g->num_edges * e_dim;
    const int blocks = (int)std::min<int64_t>(gnn_div_up(total, 256), 256 * 64);
    hipLaunchKernelGGL(unpermute_rows_kernel, dim3(blocks), dim3(256), 0, s, g->perm, g->num_edges, d_e_csr, e_dim, d_e);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

}  // extern "C"
