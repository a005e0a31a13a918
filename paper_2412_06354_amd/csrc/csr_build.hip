// COO -> CSR by destination: index range check, stable least-significant-digit radix sort of
// (dst; src, edge id), in-degree histogram (read off the runs of the sorted destinations, so
// hub nodes cost no contended atomics), exclusive scan to rowptr, and the degree-bucketed work
// lists used by the compute kernels.
//
// The paper (section 3, "Graph Data Structures") keeps topology in COO form by default and
// treats the sparse adjacency as another encoding of the same graph; this file derives the
// by-destination sparse form once per graph so that every later reduction over a node's
// neighbourhood is a contiguous segment.
#include "gnn_internal.h"

#include <algorithm>
#include <cstring>
#include <mutex>

namespace {

constexpr int kThreads = 256;

// ---------------------------------------------------------------- range check, in-degree histogram

// Range check of both index arrays; the same pass keeps a copy of the destinations in the caller's edge order
// (dst_copy may be null).
__global__ __launch_bounds__(kThreads) void check_range_kernel(const int32_t *__restrict__ src,
                                                               const int32_t *__restrict__ dst, int64_t E,
                                                               int32_t N_src, int32_t N,
                                                               int32_t *__restrict__ dst_copy,
                                                               int32_t *__restrict__ bad)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    int any_bad = 0;
    for (int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x; k < E; k += stride) {
        const int32_t s = __builtin_nontemporal_load(src + k), d = __builtin_nontemporal_load(dst + k);
        any_bad |= ((uint32_t)s >= (uint32_t)N_src) | ((uint32_t)d >= (uint32_t)N);
        if (dst_copy) __builtin_nontemporal_store(d, dst_copy + k);
    }
    if (any_bad) atomicOr(bad, 1);
}

// Row pointers straight from the sorted destinations: where the key changes from a to b at position p, the
// rows a+1 .. b start at p (rows that do not occur get the start of the next one that does); before the first
// key a = -1, after the last one the remaining rows and rowptr[N] get E.  Valid, sorted keys write every entry
// exactly once.  Keys outside [0, N) -- invalid input, reported through the range flag -- are clamped, so nothing
// outside rowptr[0 .. N] is written whatever the keys are.  Four positions per thread (one 128-bit load).
__device__ __forceinline__ void row_pointers_body(const int32_t *__restrict__ keys, int64_t E, int32_t N,
                                                  int32_t *__restrict__ rowptr)
{
    const int64_t p0 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (p0 >= E) return;
    int32_t k[5];
    k[0] = p0 > 0 ? keys[p0 - 1] : -1;
    const int cnt = (int)min((int64_t)4, E - p0);
    if (cnt == 4 && (reinterpret_cast<uintptr_t>(keys) & 15u) == 0) {
        const int4 v = *reinterpret_cast<const int4 *>(keys + p0);
        k[1] = v.x; k[2] = v.y; k[3] = v.z; k[4] = v.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) k[j + 1] = j < cnt ? keys[p0 + j] : 0;
    }
#pragma unroll
    for (int j = 0; j < 5; ++j) k[j] = min(max(k[j], -1), N - 1);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (j < cnt)
            for (int32_t r = k[j] + 1; r <= k[j + 1]; ++r) rowptr[r] = (int32_t)(p0 + j);
    if (p0 + cnt == E)
        for (int32_t r = k[cnt] + 1; r <= N; ++r) rowptr[r] = (int32_t)E;
}

__global__ __launch_bounds__(kThreads) void row_pointers_kernel(const int32_t *__restrict__ keys, int64_t E, int32_t N,
                                                                int32_t *__restrict__ rowptr)
{
    row_pointers_body(keys, E, N, rowptr);
}

// ---------------------------------------------------------------- radix sort passes

constexpr int kSortItems = 16;                       // keys per thread
constexpr int kSortTile = kThreads * kSortItems;     // keys per block
constexpr int kDigitBitsMax = 8;   // 10-bit digits (two passes at 2^20 nodes) were measured: the scatter pass takes 2.4 x as long
constexpr int kRadixMax = 1 << kDigitBitsMax;

// Per-tile digit counts, laid out [digit][tile]: an exclusive scan along each digit's row gives, for every
// (digit, tile), the number of that digit's keys in earlier tiles, and the row totals give the digits' first
// positions in the output (added up by the scatter pass itself).
constexpr int kCountThreads = 1024;
constexpr int kCountItems = kSortTile / kCountThreads;
constexpr int kCountCopies = 8;

// CHECK: the first pass over the caller's arrays also does the range check of both index arrays and keeps a copy
// of the destinations (the keys) in the caller's edge order.
template <bool CHECK>
__device__ __forceinline__ void sort_count_body(const int32_t *__restrict__ keys, int64_t n, int shift, int bits,
                                                int32_t *__restrict__ tile_counts, int num_tiles,
                                                const int32_t *__restrict__ src, int32_t N_src, int32_t N,
                                                int32_t *__restrict__ key_copy, int32_t *__restrict__ bad)
{
    // Every digit has kCountCopies counters, lane l adds to copy l % kCountCopies: lanes that hold the same digit
    // (a hub node fills many lanes of a wavefront in the later passes, whose input is sorted by the low bits)
    // spread over several LDS addresses in different banks instead of queueing on one.
    __shared__ int cnt[kRadixMax * kCountCopies];   // [digit][copy]
    const int radix = 1 << bits, mask = radix - 1;
    for (int d = threadIdx.x; d < radix * kCountCopies; d += kCountThreads) cnt[d] = 0;
    const int copy = threadIdx.x & (kCountCopies - 1);
    // A block walks over several tiles; the next tile's keys are loaded while this one's are counted.
    int key[kCountItems], next_key[kCountItems], next_src[kCountItems];
    auto load_tile = [&](int tile) {
        const int64_t base = (int64_t)tile * kSortTile;
#pragma unroll
        for (int i = 0; i < kCountItems; ++i) {
            const int64_t idx = base + i * kCountThreads + threadIdx.x;
            const bool there = tile < num_tiles && idx < n;
            next_key[i] = there ? __builtin_nontemporal_load(keys + idx) : 0;
            if constexpr (CHECK) next_src[i] = there ? __builtin_nontemporal_load(src + idx) : 0;
        }
    };
    int any_bad = 0;
    load_tile(blockIdx.x);
    for (int tile = blockIdx.x; tile < num_tiles; tile += gridDim.x) {
#pragma unroll
        for (int i = 0; i < kCountItems; ++i) {
            key[i] = next_key[i];
            if constexpr (CHECK) any_bad |= ((uint32_t)next_src[i] >= (uint32_t)N_src) | ((uint32_t)key[i] >= (uint32_t)N);
        }
        __syncthreads();   // counters are zero
        load_tile(tile + gridDim.x);
#pragma unroll
        for (int i = 0; i < kCountItems; ++i) {
            const int64_t idx = (int64_t)tile * kSortTile + i * kCountThreads + threadIdx.x;
            const bool valid = idx < n;
            const int d = (key[i] >> shift) & mask;
            if (valid) atomicAdd(&cnt[d * kCountCopies + copy], 1);
            if constexpr (CHECK)
                if (valid) __builtin_nontemporal_store(key[i], key_copy + idx);
        }
        __syncthreads();
        for (int d = threadIdx.x; d < radix; d += kCountThreads) {
            int t = 0;
#pragma unroll
            for (int q = 0; q < kCountCopies; ++q) {
                t += cnt[d * kCountCopies + q];
                cnt[d * kCountCopies + q] = 0;
            }
            tile_counts[(int64_t)d * num_tiles + tile] = t;
        }
    }
    if constexpr (CHECK)
        if (any_bad) atomicOr(bad, 1);
}

template <bool CHECK>
__global__ __launch_bounds__(kCountThreads) void sort_count_kernel(const int32_t *__restrict__ keys, int64_t n, int shift,
                                                                   int bits, int32_t *__restrict__ tile_counts,
                                                                   int num_tiles, const int32_t *__restrict__ src,
                                                                   int32_t N_src, int32_t N,
                                                                   int32_t *__restrict__ key_copy,
                                                                   int32_t *__restrict__ bad)
{
    sort_count_body<CHECK>(keys, n, shift, bits, tile_counts, num_tiles, src, N_src, N, key_copy, bad);
}

// Stable scatter of one pass.  A tile (kSortTile consecutive keys) is handled by a block of
// kScatterThreads threads, kScatterItems keys per thread; inside a tile the order is: wavefront, then
// item, then lane; key `idx` of wavefront w is tile_base + w*64*items + item*64 + lane, so this order is
// the input order.  A key's position inside the tile's digit-sorted order is
//   (keys of smaller digits in the tile) + (same-digit keys of earlier wavefronts)
//   + (same-digit keys of this wavefront in earlier items or lower lanes);
// the last term comes from ballots: the lanes holding the same digit are found bit by bit.
// Keys, values and edge ids are all loaded up front, then passed through LDS in that order in one
// phase, so that consecutive threads write consecutive global addresses (each digit of a tile is one
// contiguous run).  Many short per-thread chains (16 wavefronts x 4 items) hide the latency of the
// ranking loop better than few long ones: 145 us per pass at 20 M keys against 210 us for 4 x 16.
constexpr int kDies = 8;
constexpr int kScatterThreads = 1024;
constexpr int kScatterItems = kSortTile / kScatterThreads;
constexpr int kScatterWaves = kScatterThreads / 64;
static_assert(kScatterItems * kScatterThreads == kSortTile, "tile size");

template <int BITS>
__device__ __forceinline__ void sort_scatter_body(
    const int32_t *__restrict__ keys_in, const int32_t *__restrict__ val_in, const int32_t *__restrict__ eid_in,
    int64_t n, int shift, const int32_t *__restrict__ tile_offsets,
    const int32_t *__restrict__ digit_totals, int num_tiles,
    int32_t *__restrict__ keys_out, int32_t *__restrict__ val_out, int32_t *__restrict__ eid_out)
{
    __shared__ int wcnt[kScatterWaves * kRadixMax];   // [wavefront][digit], rows of `radix` entries
    __shared__ int dbase[kRadixMax];   // first tile-local position of each digit
    __shared__ int gbase[kRadixMax];   // global position of that element minus dbase
    __shared__ long long wave_sums[kScatterWaves];
    __shared__ int stage[3][kSortTile];
    constexpr int radix = 1 << BITS, mask = radix - 1;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // Blocks are dealt round-robin to the chip's eight dies, each with an L2 of its own.  A die gets a contiguous
    // range of tiles: neighbouring tiles' runs of one digit are neighbours in memory, and written through the
    // same L2 they merge into whole lines before they leave it.  (The grid is rounded up to a multiple of 8.)
    const int tiles_per_die = (num_tiles + kDies - 1) / kDies;
    const int tile = (int)(blockIdx.x % kDies) * tiles_per_die + (int)(blockIdx.x / kDies);
    if (tile >= num_tiles) return;
    for (int d = threadIdx.x; d < kScatterWaves * radix; d += kScatterThreads) wcnt[d] = 0;

    const int64_t tile_base = (int64_t)tile * kSortTile;
    const int64_t wbase = tile_base + (int64_t)w * 64 * kScatterItems;
    const int tile_count = (int)min((int64_t)kSortTile, n - tile_base);
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    // tile_offsets[digit][tile] counts the digit's keys in earlier tiles; the digit's first position in the whole
    // output is the sum of the smaller digits' totals, taken below in the same scan as the tile-local bases
    const bool digit_thread = (int)threadIdx.x < radix;
    const int digit_total = digit_thread ? digit_totals[threadIdx.x] : 0;
    const int digit_earlier = digit_thread ? tile_offsets[(int64_t)threadIdx.x * num_tiles + tile] : 0;
    int key[kScatterItems], val[kScatterItems], eid[kScatterItems], lpos[kScatterItems];
#pragma unroll
    for (int i = 0; i < kScatterItems; ++i) {
        const int64_t idx = wbase + i * 64 + lane;
        const bool valid = idx < n;
        key[i] = valid ? keys_in[idx] : 0;
        val[i] = valid ? val_in[idx] : 0;
        eid[i] = valid ? (eid_in ? eid_in[idx] : (int32_t)idx) : 0;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kScatterItems; ++i) {
        const int64_t idx = wbase + i * 64 + lane;
        const bool valid = idx < n;
        const int d = (key[i] >> shift) & mask;
        uint64_t peers = __ballot(valid);   // lanes of this wavefront that hold the same digit (and a key at all)
#pragma unroll
        for (int b = 0; b < BITS; ++b) {
            const int32_t x = (int32_t)((uint32_t)d << (31 - b)) >> 31;   // all ones where bit b is set
            const uint64_t m = __ballot(x != 0);
            const uint64_t xx = ((uint64_t)(uint32_t)x << 32) | (uint32_t)x;
            peers &= ~(m ^ xx);   // lanes whose bit b equals mine
        }
        const int r = __popcll(peers & lt_mask);
        // the first lane of every group takes the group's places in the wavefront's counter row (one lane per
        // digit: no two lanes share an address) and hands the old count to the others
        int before = 0;
        if (valid && r == 0) before = atomicAdd(&wcnt[w * radix + d], __popcll(peers));
        const int leader = (__ffsll((long long)peers) - 1) & 63;
        before = __shfl(before, leader, 64);
        lpos[i] = before + r;
    }
    __syncthreads();
    // per digit: offsets of the wavefronts inside the digit, digit totals -> tile-local digit bases
    int total = 0;
    if (digit_thread) {
        const int d = threadIdx.x;
#pragma unroll
        for (int q = 0; q < kScatterWaves; ++q) {
            const int c = wcnt[q * radix + d];
            wcnt[q * radix + d] = total;
            total += c;
        }
    }
    int excl, digit_first;
    {   // block-wide exclusive scan over the digits of two sums at once: the tile's counts (at most kSortTile in
        // all, the low 16 bits) and the whole input's counts (less than 2^31 in all, the bits above)
        static_assert(kSortTile < (1 << 16), "tile-local counts share a word with the global ones");
        const long long both = ((long long)digit_total << 16) | (long long)total;
        long long inc = both;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long t = __shfl_up(inc, off, 64);
            if (lane >= off) inc += t;
        }
        if (lane == 63) wave_sums[w] = inc;
        __syncthreads();
        long long base = 0;
        for (int q = 0; q < kScatterWaves; ++q)
            if (q < w) base += wave_sums[q];
        const long long before = base + inc - both;
        excl = (int)(before & 0xffff);
        digit_first = (int)(before >> 16);
    }
    if (digit_thread) {
        dbase[threadIdx.x] = excl;
        gbase[threadIdx.x] = digit_first + digit_earlier - excl;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kScatterItems; ++i) {
        const int64_t idx = wbase + i * 64 + lane;
        if (idx < n) {
            const int d = (key[i] >> shift) & mask;
            const int pos = lpos[i] + dbase[d] + wcnt[w * radix + d];
            stage[0][pos] = key[i];
            stage[1][pos] = val[i];
            stage[2][pos] = eid[i];
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kScatterItems; ++i) {
        const int s = i * kScatterThreads + threadIdx.x;
        if (s < tile_count) {
            const int k = stage[0][s];
            const int gpos = gbase[(k >> shift) & mask] + s;
            if (keys_out) keys_out[gpos] = k;
            val_out[gpos] = stage[1][s];
            eid_out[gpos] = stage[2][s];
        }
    }
}

template <int BITS>
__global__ __launch_bounds__(kScatterThreads) void sort_scatter_kernel(
    const int32_t *__restrict__ keys_in, const int32_t *__restrict__ val_in, const int32_t *__restrict__ eid_in,
    int64_t n, int shift, const int32_t *__restrict__ tile_offsets,
    const int32_t *__restrict__ digit_totals, int num_tiles,
    int32_t *__restrict__ keys_out, int32_t *__restrict__ val_out, int32_t *__restrict__ eid_out)
{
    sort_scatter_body<BITS>(keys_in, val_in, eid_in, n, shift, tile_offsets, digit_totals, num_tiles, keys_out, val_out,
                            eid_out);
}

// The digit width is a compile-time constant of the scatter kernel (its bit-by-bit matching loop is unrolled).
template <int BITS>
gnn_status launch_scatter_bits(int64_t blocks, hipStream_t stream, const int32_t *ki, const int32_t *vi, const int32_t *ei,
                               int64_t E, int shift, const int32_t *counts, const int32_t *digit_totals, int num_tiles,
                               int32_t *ko, int32_t *vo, int32_t *eo)
{
    hipLaunchKernelGGL(sort_scatter_kernel<BITS>, dim3((unsigned)blocks), dim3(kScatterThreads), 0, stream, ki, vi, ei, E,
                       shift, counts, digit_totals, num_tiles, ko, vo, eo);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status launch_scatter(int bits, int64_t blocks, hipStream_t stream, const int32_t *ki, const int32_t *vi,
                          const int32_t *ei, int64_t E, int shift, const int32_t *counts, const int32_t *digit_totals,
                          int num_tiles, int32_t *ko, int32_t *vo, int32_t *eo)
{
    switch (bits) {
    case 1: return launch_scatter_bits<1>(blocks, stream, ki, vi, ei, E, shift, counts, digit_totals, num_tiles, ko, vo, eo);
    case 2: return launch_scatter_bits<2>(blocks, stream, ki, vi, ei, E, shift, counts, digit_totals, num_tiles, ko, vo, eo);
    case 3: return launch_scatter_bits<3>(blocks, stream, ki, vi, ei, E, shift, counts, digit_totals, num_tiles, ko, vo, eo);
    case 4: return launch_scatter_bits<4>(blocks, stream, ki, vi, ei, E, shift, counts, digit_totals, num_tiles, ko, vo, eo);
    case 5: return launch_scatter_bits<5>(blocks, stream, ki, vi, ei, E, shift, counts, digit_totals, num_tiles, ko, vo, eo);
    case 6: return launch_scatter_bits<6>(blocks, stream, ki, vi, ei, E, shift, counts, digit_totals, num_tiles, ko, vo, eo);
    case 7: return launch_scatter_bits<7>(blocks, stream, ki, vi, ei, E, shift, counts, digit_totals, num_tiles, ko, vo, eo);
    case 8: return launch_scatter_bits<8>(blocks, stream, ki, vi, ei, E, shift, counts, digit_totals, num_tiles, ko, vo, eo);
    }
    return GNN_ERR_BAD_SIZE;
}

__global__ __launch_bounds__(kThreads) void iota_copy_kernel(const int32_t *__restrict__ key_in,
                                                             const int32_t *__restrict__ val_in, int64_t n,
                                                             int32_t *__restrict__ key_out,
                                                             int32_t *__restrict__ val_out,
                                                             int32_t *__restrict__ eid_out)
{
    const int64_t k = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (k < n) {
        key_out[k] = key_in[k];
        val_out[k] = val_in[k];
        eid_out[k] = (int32_t)k;
    }
}

// ---------------------------------------------------------------- work lists

// Two kernels and a small scan in between.  A block owns kListRows consecutive rows, a thread kListRowsPerThread of
// them.  Per row: is it a short row, how many wavefront pieces it needs, how many partial-result slots (pieces of
// rows made of more than one piece), is it split.  classify_rows_kernel writes what is kept per row (in-degree,
// the two degree factors of the GCN normalisation) and the block's four sums; a row-wise scan turns the sums into
// each block's first position in the four lists (and the lists' sizes); fill_lists_kernel classifies its rows again
// -- cheaper than storing and re-reading four flags per row -- scans inside the block and writes the lists.
// Everything is in row order and free of atomics, so the lists are the same on every run.
constexpr int kListRowsPerThread = 4;
constexpr int kListRows = kThreads * kListRowsPerThread;

struct RowCounts {
    long long small_split = 0;   // short rows in the low 32 bits, split rows above
    long long items_slots = 0;   // pieces in the low 32 bits, slots above
};

// Sums fit their halves: at most kListRows rows per block, and less than 2^31 / 64 + kListRows pieces.
__device__ __forceinline__ void count_row(RowCounts &c, int deg, int small_max, int chunk)
{
    const int small = deg <= small_max;
    const int items = small ? 0 : (deg + chunk - 1) / chunk;
    const int split = items > 1;
    c.small_split += (long long)small | ((long long)split << 32);
    c.items_slots += (long long)items | ((long long)(split ? items : 0) << 32);
}

// Exclusive scan of one value per thread over the block; *total receives the block's sum.
__device__ __forceinline__ long long block_exclusive_scan_i64(long long v, long long *total)
{
    __shared__ long long wave_sums[kThreads / 64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    long long inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const long long t = __shfl_up(inc, off, 64);
        if (lane >= off) inc += t;
    }
    if (lane == 63) wave_sums[w] = inc;
    __syncthreads();
    long long before = 0, all = 0;
#pragma unroll
    for (int q = 0; q < kThreads / 64; ++q) {
        const long long t = wave_sums[q];
        if (q < w) before += t;
        all += t;
    }
    __syncthreads();   // wave_sums is written again by the next call
    *total = all;
    return before + inc - v;
}

// Row pointers of the thread's rows: rp[i] = rowptr[r0 + i] for r0 + i <= N (0 beyond).
__device__ __forceinline__ void load_row_pointers(const int32_t *__restrict__ rowptr, int32_t N, int64_t r0,
                                                  int32_t (&rp)[kListRowsPerThread + 1])
{
#pragma unroll
    for (int i = 0; i <= kListRowsPerThread; ++i) rp[i] = (r0 + i <= N) ? rowptr[r0 + i] : 0;
}

__device__ __forceinline__ void classify_rows_body(const int32_t *__restrict__ rowptr, int32_t N, int32_t small_max,
                                                   int32_t chunk, const int32_t *__restrict__ bad,
                                                   int32_t *__restrict__ indeg, float *__restrict__ dinv_loop,
                                                   float *__restrict__ dinv_plain, int32_t *__restrict__ block_sums,
                                                   int num_blocks)
{
    const int64_t r0 = (int64_t)blockIdx.x * kListRows + (int64_t)threadIdx.x * kListRowsPerThread;
    // invalid input (the build will fail with an error): the row pointers mean nothing, every row counts as empty
    const bool invalid = bad[0] != 0;
    int32_t rp[kListRowsPerThread + 1];
    load_row_pointers(rowptr, N, r0, rp);
    RowCounts c;
#pragma unroll
    for (int i = 0; i < kListRowsPerThread; ++i) {
        const int64_t r = r0 + i;
        if (r < N) {
            const int32_t deg = invalid ? 0 : rp[i + 1] - rp[i];
            indeg[r] = deg;
            // the two degree factors of the GCN normalisation, kept with the graph
            dinv_loop[r] = 1.0f / sqrtf((float)(deg + 1));
            dinv_plain[r] = deg > 0 ? 1.0f / sqrtf((float)deg) : 0.0f;
            count_row(c, deg, small_max, chunk);
        }
    }
    long long ss, is;
    (void)block_exclusive_scan_i64(c.small_split, &ss);
    (void)block_exclusive_scan_i64(c.items_slots, &is);
    if (threadIdx.x == 0) {   // [list][block]: small rows, pieces, slots, split rows
        block_sums[0 * (int64_t)num_blocks + blockIdx.x] = (int32_t)(ss & 0xffffffffll);
        block_sums[1 * (int64_t)num_blocks + blockIdx.x] = (int32_t)(is & 0xffffffffll);
        block_sums[2 * (int64_t)num_blocks + blockIdx.x] = (int32_t)(is >> 32);
        block_sums[3 * (int64_t)num_blocks + blockIdx.x] = (int32_t)(ss >> 32);
    }
}

__global__ __launch_bounds__(kThreads) void classify_rows_kernel(const int32_t *__restrict__ rowptr, int32_t N,
                                                                 int32_t small_max, int32_t chunk,
                                                                 const int32_t *__restrict__ bad,
                                                                 int32_t *__restrict__ indeg,
                                                                 float *__restrict__ dinv_loop,
                                                                 float *__restrict__ dinv_plain,
                                                                 int32_t *__restrict__ block_sums, int num_blocks)
{
    classify_rows_body(rowptr, N, small_max, chunk, bad, indeg, dinv_loop, dinv_plain, block_sums, num_blocks);
}

// block_first: block_sums after the exclusive scan along each of its four rows; list_sizes: the four row totals.
// info[0] = the range flag, info[1 .. 4] = the sizes of the lists (one host read-back for all five).
__device__ __forceinline__ void fill_lists_body(
    const int32_t *__restrict__ rowptr, int32_t N, int32_t small_max, int32_t chunk, const int32_t *__restrict__ bad,
    const int32_t *__restrict__ block_first, int num_blocks, const int32_t *__restrict__ list_sizes,
    int32_t *__restrict__ small_rows, int32_t *__restrict__ item_row, int32_t *__restrict__ item_start,
    int32_t *__restrict__ item_slot, int32_t *__restrict__ split_rows, int32_t *__restrict__ split_slot0,
    int32_t *__restrict__ info)
{
    const bool invalid = bad[0] != 0;
    if (blockIdx.x == 0 && threadIdx.x < 4) info[1 + threadIdx.x] = list_sizes[threadIdx.x];
    if (blockIdx.x == 0 && threadIdx.x == 0) info[0] = invalid ? 1 : 0;
    if (invalid) return;   // the whole grid leaves: the lists were sized for empty rows
    const int64_t r0 = (int64_t)blockIdx.x * kListRows + (int64_t)threadIdx.x * kListRowsPerThread;
    int32_t rp[kListRowsPerThread + 1];
    load_row_pointers(rowptr, N, r0, rp);
    RowCounts c;
#pragma unroll
    for (int i = 0; i < kListRowsPerThread; ++i)
        if (r0 + i < N) count_row(c, rp[i + 1] - rp[i], small_max, chunk);
    long long unused;
    const long long ss = block_exclusive_scan_i64(c.small_split, &unused);
    const long long is = block_exclusive_scan_i64(c.items_slots, &unused);
    int32_t p_small = block_first[0 * (int64_t)num_blocks + blockIdx.x] + (int32_t)(ss & 0xffffffffll);
    int32_t p_item = block_first[1 * (int64_t)num_blocks + blockIdx.x] + (int32_t)(is & 0xffffffffll);
    int32_t p_slot = block_first[2 * (int64_t)num_blocks + blockIdx.x] + (int32_t)(is >> 32);
    int32_t p_split = block_first[3 * (int64_t)num_blocks + blockIdx.x] + (int32_t)(ss >> 32);
#pragma unroll
    for (int i = 0; i < kListRowsPerThread; ++i) {
        const int64_t r = r0 + i;
        if (r >= N) break;
        const int32_t start = rp[i], deg = rp[i + 1] - rp[i];
        if (deg <= small_max) {
            small_rows[p_small++] = (int32_t)r;
            continue;
        }
        const int items = (deg + chunk - 1) / chunk;
        if (items == 1) {
            item_row[p_item] = (int32_t)r;
            item_start[p_item] = start;
            item_slot[p_item] = -1;
            ++p_item;
            continue;
        }
        split_rows[p_split] = (int32_t)r;
        split_slot0[p_split] = p_slot;
        ++p_split;
        for (int q = 0; q < items; ++q) {
            item_row[p_item + q] = (int32_t)r;
            item_start[p_item + q] = start + q * chunk;
            item_slot[p_item + q] = p_slot + q;
        }
        p_item += items;
        p_slot += items;
    }
}

__global__ __launch_bounds__(kThreads) void fill_lists_kernel(
    const int32_t *__restrict__ rowptr, int32_t N, int32_t small_max, int32_t chunk, const int32_t *__restrict__ bad,
    const int32_t *__restrict__ block_first, int num_blocks, const int32_t *__restrict__ list_sizes,
    int32_t *__restrict__ small_rows, int32_t *__restrict__ item_row, int32_t *__restrict__ item_start,
    int32_t *__restrict__ item_slot, int32_t *__restrict__ split_rows, int32_t *__restrict__ split_slot0,
    int32_t *__restrict__ info)
{
    fill_lists_body(rowptr, N, small_max, chunk, bad, block_first, num_blocks, list_sizes, small_rows, item_row,
                    item_start, item_slot, split_rows, split_slot0, info);
}

// ---------------------------------------------------------------- the same kernels over a batch of builds

// One build of a batch (gnn_build_csr_batch: the snapshots of a temporal graph over one node set): what differs
// from build to build.  The kernels below are the kernels above with blockIdx.y naming the build; a launch covers
// every build of the batch, so the launch count does not grow with the number of snapshots.
struct BuildJob {
    const int32_t *src, *dst;   // the caller's edge list
    int64_t E;
    int32_t num_tiles, small_max, chunk, pad;
    int32_t *kb, *vb, *eb, *counts, *digit_totals, *block_sums, *list_sizes, *flag;   // temporaries of this build
    int32_t *rowptr, *indeg, *colidx, *perm, *rowidx, *dst_coo;                       // arrays of its graph
    float *dinv_loop, *dinv_plain;
    int32_t *small_rows, *item_row, *item_start, *item_slot, *split_rows, *split_slot0;
};

// The three arrays a sort pass reads or writes: 0 = the caller's (dst, src, edge id = position), 1 = the
// temporaries, 2 = the arrays the graph keeps.
struct SortArrays {
    int32_t *k, *v, *e;
};

__device__ __forceinline__ SortArrays sort_arrays(const BuildJob &j, int sel)
{
    if (sel == 0) return {const_cast<int32_t *>(j.dst), const_cast<int32_t *>(j.src), nullptr};   // only ever read
    if (sel == 1) return {j.kb, j.vb, j.eb};
    return {j.rowidx, j.colidx, j.perm};
}

template <bool CHECK>
__global__ __launch_bounds__(kCountThreads) void sort_count_batch_kernel(const BuildJob *__restrict__ jobs, int in_sel,
                                                                         int shift, int bits, int32_t N)
{
    const BuildJob j = jobs[blockIdx.y];
    const SortArrays in = sort_arrays(j, in_sel);
    sort_count_body<CHECK>(in.k, j.E, shift, bits, j.counts, j.num_tiles, j.src, N, N, j.dst_coo, j.flag);
}

template <int BITS>
__global__ __launch_bounds__(kScatterThreads) void sort_scatter_batch_kernel(const BuildJob *__restrict__ jobs,
                                                                             int in_sel, int out_sel, int shift)
{
    const BuildJob j = jobs[blockIdx.y];
    const SortArrays in = sort_arrays(j, in_sel), out = sort_arrays(j, out_sel);
    sort_scatter_body<BITS>(in.k, in.v, in.e, j.E, shift, j.counts, j.digit_totals, j.num_tiles, out.k, out.v, out.e);
}

__global__ __launch_bounds__(kThreads) void row_pointers_batch_kernel(const BuildJob *__restrict__ jobs, int32_t N)
{
    const BuildJob j = jobs[blockIdx.y];
    row_pointers_body(j.rowidx, j.E, N, j.rowptr);
}

__global__ __launch_bounds__(kThreads) void classify_rows_batch_kernel(const BuildJob *__restrict__ jobs, int32_t N,
                                                                       int num_blocks)
{
    const BuildJob j = jobs[blockIdx.y];
    classify_rows_body(j.rowptr, N, j.small_max, j.chunk, j.flag, j.indeg, j.dinv_loop, j.dinv_plain, j.block_sums,
                       num_blocks);
}

__global__ __launch_bounds__(kThreads) void fill_lists_batch_kernel(const BuildJob *__restrict__ jobs, int32_t N,
                                                                    int num_blocks)
{
    const BuildJob j = jobs[blockIdx.y];
    fill_lists_body(j.rowptr, N, j.small_max, j.chunk, j.flag, j.block_sums, num_blocks, j.list_sizes, j.small_rows,
                    j.item_row, j.item_start, j.item_slot, j.split_rows, j.split_slot0, j.flag + 8);
}

template <int BITS>
gnn_status launch_scatter_batch_bits(dim3 grid, hipStream_t stream, const BuildJob *jobs, int in_sel, int out_sel,
                                     int shift)
{
    hipLaunchKernelGGL(sort_scatter_batch_kernel<BITS>, grid, dim3(kScatterThreads), 0, stream, jobs, in_sel, out_sel,
                       shift);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

gnn_status launch_scatter_batch(int bits, dim3 grid, hipStream_t stream, const BuildJob *jobs, int in_sel, int out_sel,
                                int shift)
{
    switch (bits) {
    case 1: return launch_scatter_batch_bits<1>(grid, stream, jobs, in_sel, out_sel, shift);
    case 2: return launch_scatter_batch_bits<2>(grid, stream, jobs, in_sel, out_sel, shift);
    case 3: return launch_scatter_batch_bits<3>(grid, stream, jobs, in_sel, out_sel, shift);
    case 4: return launch_scatter_batch_bits<4>(grid, stream, jobs, in_sel, out_sel, shift);
    case 5: return launch_scatter_batch_bits<5>(grid, stream, jobs, in_sel, out_sel, shift);
    case 6: return launch_scatter_batch_bits<6>(grid, stream, jobs, in_sel, out_sel, shift);
    case 7: return launch_scatter_batch_bits<7>(grid, stream, jobs, in_sel, out_sel, shift);
    case 8: return launch_scatter_batch_bits<8>(grid, stream, jobs, in_sel, out_sel, shift);
    }
    return GNN_ERR_BAD_SIZE;
}

__global__ __launch_bounds__(kThreads) void permute_rows_kernel(const int32_t *__restrict__ perm, int64_t E,
                                                                const float *__restrict__ e, int32_t e_dim,
                                                                float *__restrict__ e_csr)
{
    const int64_t total = E * e_dim;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t q = (int64_t)blockIdx.x * kThreads + threadIdx.x; q < total; q += stride) {
        const int64_t p = q / e_dim;
        const int32_t c = (int32_t)(q - p * e_dim);
        e_csr[q] = e[(int64_t)perm[p] * e_dim + c];
    }
}

int ceil_log2(uint32_t n)
{
    int b = 0;
    while ((1ull << b) < n) ++b;
    return b;
}

// The arrays of a destroyed graph are kept for the next build: one block per process (the larger one wins), so
// that a loop which builds a graph per mini-batch and destroys the previous one neither allocates nor frees in
// steady state (an allocation plus a free cost about as much as the kernels of a 20 M-edge build).  A build takes
// the block if it is on the current device, large enough and at most twice what it needs.
// gnn_release_cached_memory() frees it.
struct slab_cache {
    std::mutex mu;
    void *ptr = nullptr;
    size_t bytes = 0;
    int device = -1;
};
slab_cache g_slab_cache;

// Offers a block that is no longer used to the cache; returns the block to free (the offered one, the smaller one
// it replaces, or none).
void *slab_cache_put(void *ptr, size_t bytes, int device)
{
    if (!ptr) return nullptr;
    std::lock_guard<std::mutex> lock(g_slab_cache.mu);
    slab_cache &c = g_slab_cache;
    if (c.ptr && c.bytes >= bytes) return ptr;
    void *drop = c.ptr;
    c.ptr = ptr;
    c.bytes = bytes;
    c.device = device;
    return drop;
}

// Takes the cached block if it is on this device, large enough and at most twice what is needed.
bool slab_cache_take(size_t bytes, int device, void **ptr, size_t *got_bytes)
{
    std::lock_guard<std::mutex> lock(g_slab_cache.mu);
    slab_cache &c = g_slab_cache;
    if (!(c.ptr && c.device == device && c.bytes >= bytes && c.bytes / 2 <= bytes)) return false;
    *ptr = c.ptr;
    *got_bytes = c.bytes;
    c.ptr = nullptr;
    c.bytes = 0;
    c.device = -1;
    return true;
}

void free_graph_arrays(gnn_graph *g)
{
    void *drop = nullptr;
    if (g->shared) {   // one allocation for a batch of graphs: given up with the last of them
        if (g->shared->refs.fetch_sub(1) == 1) {
            drop = slab_cache_put(g->shared->ptr, g->shared->bytes, g->shared->device);
            delete g->shared;
        }
        g->shared = nullptr;
    } else if (g->slab) {
        drop = slab_cache_put(g->slab, g->slab_bytes, g->device);
    }
    if (drop) (void)hipFree(drop);
    if (g->own_scratch) (void)hipFree(g->own_scratch);
    gnn_route_free(g);
    g->slab = nullptr;
    g->slab_bytes = 0;
    g->scratch = nullptr;
    g->scratch_floats = 0;
    g->own_scratch = nullptr;
}

// Carves 256-byte aligned int32 arrays out of one device allocation.
struct slab_plan {
    size_t bytes = 0;
    size_t add(size_t count) {
        const size_t off = bytes;
        bytes += ((count ? count : 1) * sizeof(int32_t) + 255) & ~(size_t)255;
        return off;
    }
};

gnn_status slab_alloc(void **out, size_t bytes)
{
    *out = nullptr;
    if (hipMalloc(out, bytes ? bytes : 256) != hipSuccess) {
        (void)hipGetLastError();
        *out = nullptr;
        return GNN_ERR_ALLOC;
    }
    return GNN_OK;
}

gnn_status graph_slab_acquire(gnn_graph *g, size_t bytes)
{
    int dev = 0;
    GNN_HIP(hipGetDevice(&dev));
    g->device = dev;
    if (slab_cache_take(bytes, dev, &g->slab, &g->slab_bytes)) return GNN_OK;
    GNN_TRY(slab_alloc(&g->slab, bytes));
    g->slab_bytes = bytes ? bytes : 256;
    return GNN_OK;
}

// The temporaries of a build (sort buffers, counts, flags) are kept between calls: one grow-only device
// buffer per process, lent to one build at a time (a build ends with a stream synchronisation, so the buffer
// is idle when it is handed back).  A build that finds it lent out, on another device, or that needs more
// than kTempCacheLimit allocates and frees its own.  gnn_release_cached_memory() frees it.
constexpr size_t kTempCacheLimit = (size_t)8 << 30;

struct temp_cache {
    std::mutex mu;
    void *ptr = nullptr;
    size_t bytes = 0;
    int device = -1;
    bool lent = false;
};
temp_cache g_temp_cache;

struct temp_lease {
    void *ptr = nullptr;
    bool cached = false;
    ~temp_lease()
    {
        if (!ptr) return;
        if (cached) {
            std::lock_guard<std::mutex> lock(g_temp_cache.mu);
            g_temp_cache.lent = false;
        } else {
            (void)hipFree(ptr);
        }
    }
};

gnn_status temp_acquire(temp_lease *lease, size_t bytes)
{
    int dev = 0;
    GNN_HIP(hipGetDevice(&dev));
    {
        std::lock_guard<std::mutex> lock(g_temp_cache.mu);
        temp_cache &c = g_temp_cache;
        if (!c.lent && bytes <= kTempCacheLimit) {
            if (c.ptr && (c.device != dev || c.bytes < bytes)) {
                (void)hipFree(c.ptr);   // nobody holds it: replace by a larger one / one on this device
                c.ptr = nullptr;
                c.bytes = 0;
            }
            if (!c.ptr) {
                const size_t want = bytes + bytes / 8;   // some head-room for the next, slightly larger graph
                if (hipMalloc(&c.ptr, want) != hipSuccess) {
                    (void)hipGetLastError();
                    c.ptr = nullptr;
                    return GNN_ERR_ALLOC;
                }
                c.bytes = want;
                c.device = dev;
            }
            c.lent = true;
            lease->ptr = c.ptr;
            lease->cached = true;
            return GNN_OK;
        }
    }
    lease->cached = false;
    return slab_alloc(&lease->ptr, bytes);
}

int32_t *at(void *slab, size_t off) { return reinterpret_cast<int32_t *>(static_cast<char *>(slab) + off); }

// Where the arrays a graph keeps lie inside its allocation.
struct graph_layout {
    size_t o_rowptr, o_indeg, o_colidx, o_perm, o_rowidx, o_dstcoo, o_small, o_irow, o_istart, o_islot, o_srows, o_sslot,
        o_dinv1, o_dinv0, o_scratch;
    size_t scratch_floats;
    size_t bytes;
};

graph_layout plan_graph(int64_t E, int32_t N, int32_t chunk)
{
    const size_t np1 = (size_t)N + 1;
    // Upper bounds of the work-list sizes, so that everything the graph keeps is one allocation made
    // before any kernel runs: a row is short or gives ceil(deg / chunk) pieces.
    const size_t max_items = (size_t)std::min<int64_t>(N, E) + (size_t)(E / chunk) + 1;
    const size_t max_split = (size_t)(E / chunk) + 1;
    // A split row has more than `chunk` edges and ceil(deg / chunk) <= 2 deg / chunk pieces: at most 2 E / chunk
    // slots in all.  The scratch the compute calls share is sized for that bound at the default feature width, as a
    // part of the slab, so that no compute call ever allocates (wider features: gnn_graph_reserve).
    const size_t max_slots = 2 * (size_t)(E / chunk) + 1;
    graph_layout L{};
    L.scratch_floats = gnn_scratch_floats((int64_t)max_slots, N, kDefaultReservedFeatDim, 0);
    slab_plan pa;
    L.o_rowptr = pa.add(np1); L.o_indeg = pa.add(N); L.o_colidx = pa.add(E); L.o_perm = pa.add(E);
    L.o_rowidx = pa.add(E); L.o_dstcoo = pa.add(E); L.o_small = pa.add(N); L.o_irow = pa.add(max_items);
    L.o_istart = pa.add(max_items); L.o_islot = pa.add(max_items); L.o_srows = pa.add(max_split);
    L.o_sslot = pa.add(max_split); L.o_dinv1 = pa.add(N); L.o_dinv0 = pa.add(N);
    L.o_scratch = pa.add(L.scratch_floats);
    L.bytes = pa.bytes;
    return L;
}

void bind_graph(gnn_graph *g, void *base, const graph_layout &L)
{
    g->rowptr = at(base, L.o_rowptr);
    g->indeg = at(base, L.o_indeg);
    g->colidx = at(base, L.o_colidx);
    g->perm = at(base, L.o_perm);
    g->rowidx = at(base, L.o_rowidx);
    g->dst_coo = at(base, L.o_dstcoo);
    g->dinv_loop = reinterpret_cast<float *>(at(base, L.o_dinv1));
    g->dinv_plain = reinterpret_cast<float *>(at(base, L.o_dinv0));
    g->small_rows = at(base, L.o_small);
    g->item_row = at(base, L.o_irow);
    g->item_start = at(base, L.o_istart);
    g->item_slot = at(base, L.o_islot);
    g->split_rows = at(base, L.o_srows);
    g->split_slot0 = at(base, L.o_sslot);
    g->scratch = reinterpret_cast<float *>(at(base, L.o_scratch));
    g->scratch_floats = L.scratch_floats;
}

// Temporaries of one build: sort ping-pong buffers, per-tile digit counts, block sums of the work lists.
struct temp_layout {
    size_t o_kb, o_vb, o_eb, o_counts, o_dtot, o_bsum, o_sizes;
    size_t bytes;
    int list_blocks;
    int64_t num_tiles;
};

temp_layout plan_temp(int64_t E, int32_t N)
{
    temp_layout T{};
    T.num_tiles = gnn_div_up(E, kSortTile);
    T.list_blocks = (int)gnn_div_up(N, kListRows);
    slab_plan pt;
    T.o_kb = pt.add(E); T.o_vb = pt.add(E); T.o_eb = pt.add(E);
    T.o_counts = pt.add((size_t)T.num_tiles * kRadixMax); T.o_dtot = pt.add(kRadixMax);
    T.o_bsum = pt.add(4 * (size_t)T.list_blocks); T.o_sizes = pt.add(4);
    T.bytes = pt.bytes;
    return T;
}

constexpr int kFlagInts = 64;   // per build: [0] the range flag, [8 .. 12] what is read back (flag + four list sizes)

// Enqueues every kernel of one build.  d_flag: kFlagInts zeroed ints; d_flag[8 .. 12] are filled for the host.
gnn_status enqueue_build(const int32_t *d_src, const int32_t *d_dst, int64_t E, int32_t N, hipStream_t stream,
                         gnn_graph *g, char *ts, const temp_layout &T, int32_t *d_flag)
{
    const size_t np1 = (size_t)N + 1;
    const int64_t num_tiles = T.num_tiles;
    const int list_blocks = T.list_blocks;
    int32_t *kb = at(ts, T.o_kb), *vb = at(ts, T.o_vb), *eb = at(ts, T.o_eb), *counts = at(ts, T.o_counts),
            *digit_totals = at(ts, T.o_dtot), *block_sums = at(ts, T.o_bsum), *list_sizes = at(ts, T.o_sizes);

    // ---- the index range check and the copy of the destinations in edge order ride on the first counting
    //      pass of the sort.  The flag is read back at the end; nothing below indexes with an unchecked node id:
    //      the sort only uses masked digits, the row-pointer kernel clamps its keys and the work-list kernels do
    //      nothing once the flag is set.

    // ---- stable radix sort by destination
    if (E > 0) {
        const int key_bits = ceil_log2((uint32_t)N);
        if (key_bits == 0) {   // one node: nothing to sort
            const int cblocks = (int)std::min<int64_t>(gnn_div_up(E, kThreads), 256 * 16);
            hipLaunchKernelGGL(check_range_kernel, dim3(cblocks), dim3(kThreads), 0, stream, d_src, d_dst, E,
                               g->num_src_nodes, N, g->dst_coo, d_flag);
            GNN_LAUNCH_CHECK();
            const int blocks = (int)gnn_div_up(E, kThreads);
            hipLaunchKernelGGL(iota_copy_kernel, dim3(blocks), dim3(kThreads), 0, stream, d_dst, d_src, E, g->rowidx,
                               g->colidx, g->perm);
            GNN_LAUNCH_CHECK();
        } else {
            const int passes = (key_bits + kDigitBitsMax - 1) / kDigitBitsMax;
            const int bits = (key_bits + passes - 1) / passes;
            // Ping-pong between (kb, vb, eb) and the arrays the graph keeps, arranged so that
            // the last pass writes into the graph's arrays.
            int32_t *bufk[2] = {kb, g->rowidx}, *bufv[2] = {vb, g->colidx}, *bufe[2] = {eb, g->perm};
            int dst_sel = (passes % 2 == 1) ? 1 : 0;   // buffer written by the first pass
            const int32_t *ki = d_dst, *vi = d_src, *ei = nullptr;
            for (int p = 0; p < passes; ++p) {
                const int shift = p * bits;
                const dim3 cgrid((unsigned)std::min<int64_t>(num_tiles, 1024));
                if (p == 0)   // the pass over the caller's arrays: range check and edge-order copy of dst ride along
                    hipLaunchKernelGGL(sort_count_kernel<true>, cgrid, dim3(kCountThreads), 0, stream, ki, E, shift, bits,
                                       counts, (int)num_tiles, d_src, g->num_src_nodes, N, g->dst_coo, d_flag);
                else
                    hipLaunchKernelGGL(sort_count_kernel<false>, cgrid, dim3(kCountThreads), 0, stream, ki, E, shift, bits,
                                       counts, (int)num_tiles, (const int32_t *)nullptr, 0, 0, (int32_t *)nullptr,
                                       (int32_t *)nullptr);
                GNN_LAUNCH_CHECK();
                GNN_TRY(gnn_scan_rows_exclusive_i32(counts, 1 << bits, num_tiles, digit_totals, stream));
                GNN_TRY(launch_scatter(bits, gnn_div_up(num_tiles, kDies) * kDies, stream, ki, vi, ei, E, shift, counts,
                                       digit_totals, (int)num_tiles, bufk[dst_sel], bufv[dst_sel], bufe[dst_sel]));
                ki = bufk[dst_sel];
                vi = bufv[dst_sel];
                ei = bufe[dst_sel];
                dst_sel ^= 1;
            }
        }
        // ---- row pointers from the runs of the sorted destinations
        hipLaunchKernelGGL(row_pointers_kernel, dim3((unsigned)gnn_div_up(gnn_div_up(E, 4), kThreads)), dim3(kThreads), 0,
                           stream, g->rowidx, E, N, g->rowptr);
        GNN_LAUNCH_CHECK();
    } else {
        GNN_HIP(hipMemsetAsync(g->rowptr, 0, np1 * sizeof(int32_t), stream));
    }

    // ---- work lists (positions from scans; sizes are read back afterwards)
    hipLaunchKernelGGL(classify_rows_kernel, dim3(list_blocks), dim3(kThreads), 0, stream, g->rowptr, N, g->small_max,
                       g->chunk, d_flag, g->indeg, g->dinv_loop, g->dinv_plain, block_sums, list_blocks);
    GNN_LAUNCH_CHECK();
    GNN_TRY(gnn_scan_rows_exclusive_i32(block_sums, 4, list_blocks, list_sizes, stream));
    hipLaunchKernelGGL(fill_lists_kernel, dim3(list_blocks), dim3(kThreads), 0, stream, g->rowptr, N, g->small_max,
                       g->chunk, d_flag, block_sums, list_blocks, list_sizes, g->small_rows, g->item_row,
                       g->item_start, g->item_slot, g->split_rows, g->split_slot0, d_flag + 8);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

// Enqueues the kernels of a whole batch of builds over one node set (N > 1): every launch covers all builds.
// d_jobs / d_count_scans / d_list_scans: device copies of the job tables (num_jobs entries each).
gnn_status enqueue_build_batch(const BuildJob *d_jobs, const gnn_scan_job *d_count_scans,
                               const gnn_scan_job *d_list_scans, int num_jobs, int64_t max_edges, int32_t N,
                               hipStream_t stream)
{
    const int key_bits = ceil_log2((uint32_t)N);
    const int passes = (key_bits + kDigitBitsMax - 1) / kDigitBitsMax;
    const int bits = (key_bits + passes - 1) / passes;
    const int64_t max_tiles = gnn_div_up(max_edges, kSortTile);
    const int list_blocks = (int)gnn_div_up(N, kListRows);
    constexpr int kGroup = 32768;   // builds per launch (the grid's second dimension)
    for (int first = 0; first < num_jobs; first += kGroup) {
        const unsigned count = (unsigned)std::min(kGroup, num_jobs - first);
        const BuildJob *jobs = d_jobs + first;
        if (max_edges > 0) {
            // as in a single build: ping-pong between the temporaries (1) and the graph's arrays (2), arranged so
            // that the last pass writes into the graph's arrays
            int in_sel = 0, out_sel = (passes % 2 == 1) ? 2 : 1;
            for (int p = 0; p < passes; ++p) {
                const int shift = p * bits;
                const dim3 cgrid((unsigned)std::min<int64_t>(max_tiles, 1024), count);
                if (p == 0)
                    hipLaunchKernelGGL(sort_count_batch_kernel<true>, cgrid, dim3(kCountThreads), 0, stream, jobs, in_sel,
                                       shift, bits, N);
                else
                    hipLaunchKernelGGL(sort_count_batch_kernel<false>, cgrid, dim3(kCountThreads), 0, stream, jobs, in_sel,
                                       shift, bits, N);
                GNN_LAUNCH_CHECK();
                GNN_TRY(gnn_scan_rows_exclusive_i32_jobs(d_count_scans + first, (int)count, 1 << bits, stream));
                const dim3 sgrid((unsigned)(gnn_div_up(max_tiles, kDies) * kDies), count);
                GNN_TRY(launch_scatter_batch(bits, sgrid, stream, jobs, in_sel, out_sel, shift));
                in_sel = out_sel;
                out_sel = (out_sel == 1) ? 2 : 1;
            }
            const dim3 rgrid((unsigned)gnn_div_up(gnn_div_up(max_edges, 4), kThreads), count);
            hipLaunchKernelGGL(row_pointers_batch_kernel, rgrid, dim3(kThreads), 0, stream, jobs, N);
            GNN_LAUNCH_CHECK();
        }
        const dim3 lgrid((unsigned)list_blocks, count);
        hipLaunchKernelGGL(classify_rows_batch_kernel, lgrid, dim3(kThreads), 0, stream, jobs, N, list_blocks);
        GNN_LAUNCH_CHECK();
        GNN_TRY(gnn_scan_rows_exclusive_i32_jobs(d_list_scans + first, (int)count, 4, stream));
        hipLaunchKernelGGL(fill_lists_batch_kernel, lgrid, dim3(kThreads), 0, stream, jobs, N, list_blocks);
        GNN_LAUNCH_CHECK();
    }
    return GNN_OK;
}

void take_list_sizes(gnn_graph *g, const int32_t *h_info)
{
    g->n_small = h_info[1];
    g->n_items = h_info[2];
    g->n_slots = h_info[3];
    g->n_split = h_info[4];
}

gnn_status build_impl(const int32_t *d_src, const int32_t *d_dst, int64_t E, int32_t N, hipStream_t stream,
                      gnn_graph *g)
{
    const graph_layout L = plan_graph(E, N, g->chunk);
    GNN_TRY(graph_slab_acquire(g, L.bytes));
    bind_graph(g, g->slab, L);

    // ---- temporaries: one buffer, normally the cached one; the flags sit in front of it
    const temp_layout T = plan_temp(E, N);
    const size_t flag_bytes = 256;
    static_assert(kFlagInts * sizeof(int32_t) == 256, "flag block");
    temp_lease tmp;
    GNN_TRY(temp_acquire(&tmp, flag_bytes + T.bytes));
    char *ts = static_cast<char *>(tmp.ptr);
    int32_t *d_flag = reinterpret_cast<int32_t *>(ts);
    GNN_HIP(hipMemsetAsync(d_flag, 0, flag_bytes, stream));
    GNN_TRY(enqueue_build(d_src, d_dst, E, N, stream, g, ts + flag_bytes, T, d_flag));
    int32_t h_info[5] = {0, 0, 0, 0, 0};
    GNN_HIP(hipMemcpyAsync(h_info, d_flag + 8, sizeof(h_info), hipMemcpyDeviceToHost, stream));
    GNN_HIP(hipStreamSynchronize(stream));   // everything has run: temporaries may be freed on return
    if (h_info[0]) return GNN_ERR_INDEX_RANGE;
    take_list_sizes(g, h_info);
    return GNN_OK;
}

// Default scheduling thresholds (both given as 0) and their validation.
gnn_status resolve_thresholds(int64_t num_edges, int32_t *small_max_degree, int32_t *chunk_edges)
{
    if (*small_max_degree == 0 && *chunk_edges == 0) *small_max_degree = 16;
    if (*chunk_edges == 0) {
        // long pieces amortise the per-piece overhead on big graphs; on small ones a hub row has to be cut
        // finer or its few wavefronts become the tail of the launch (measured: 256 at E = 1 M, 1024 at E >= 20 M)
        *chunk_edges = num_edges >= (int64_t)1024 * 16384 ? 1024 : num_edges >= (int64_t)512 * 16384 ? 512 : 256;
    }
    if (*small_max_degree < 0 || *small_max_degree > 64) return GNN_ERR_BAD_SIZE;
    if (*chunk_edges < 64 || *chunk_edges > 65536 || *chunk_edges % 64 != 0) return GNN_ERR_BAD_SIZE;
    return GNN_OK;
}

}  // namespace

extern "C" {

static gnn_status build_checked(const int32_t *d_src, const int32_t *d_dst, int64_t num_edges, int32_t num_src_nodes,
                                int32_t num_nodes, bool bipartite, int32_t small_max_degree, int32_t chunk_edges,
                                void *stream, gnn_graph **out_graph)
{
    if (!out_graph) return GNN_ERR_NULL;
    *out_graph = nullptr;
    if (num_nodes <= 0 || num_src_nodes <= 0 || num_edges < 0 || num_edges >= (1ll << 31)) return GNN_ERR_BAD_SIZE;
    if (num_edges > 0 && (!d_src || !d_dst)) return GNN_ERR_NULL;
    GNN_TRY(resolve_thresholds(num_edges, &small_max_degree, &chunk_edges));

    gnn_graph *g = new (std::nothrow) gnn_graph();
    if (!g) return GNN_ERR_ALLOC;
    g->num_nodes = num_nodes;
    g->num_src_nodes = num_src_nodes;
    g->bipartite = bipartite;
    g->num_edges = num_edges;
    g->small_max = small_max_degree;
    g->chunk = chunk_edges;
    gnn_status st = build_impl(d_src, d_dst, num_edges, num_nodes, static_cast<hipStream_t>(stream), g);
    if (st != GNN_OK) {
        (void)hipStreamSynchronize(static_cast<hipStream_t>(stream));
        free_graph_arrays(g);
        delete g;
        return st;
    }
    *out_graph = g;
    return GNN_OK;
}

gnn_status gnn_build_csr_ex(const int32_t *d_src, const int32_t *d_dst, int64_t num_edges, int32_t num_nodes,
                            int32_t small_max_degree, int32_t chunk_edges, void *stream, gnn_graph **out_graph)
{
    return build_checked(d_src, d_dst, num_edges, num_nodes, num_nodes, false, small_max_degree, chunk_edges, stream,
                         out_graph);
}

gnn_status gnn_build_csr_bipartite(const int32_t *d_src, const int32_t *d_dst, int64_t num_edges,
                                   int32_t num_src_nodes, int32_t num_dst_nodes, void *stream, gnn_graph **out_graph)
{
    return build_checked(d_src, d_dst, num_edges, num_src_nodes, num_dst_nodes, true, 0, 0, stream, out_graph);
}

gnn_status gnn_build_csr(const int32_t *d_src, const int32_t *d_dst, int64_t num_edges, int32_t num_nodes,
                         void *stream, gnn_graph **out_graph)
{
    return gnn_build_csr_ex(d_src, d_dst, num_edges, num_nodes, 0, 0, stream, out_graph);
}

gnn_status gnn_build_csr_batch(int32_t num_snapshots, const int32_t *const *d_src, const int32_t *const *d_dst,
                               const int64_t *num_edges, int32_t num_nodes, void *stream, gnn_graph **out_graphs)
{
    if (!out_graphs) return GNN_ERR_NULL;
    if (num_snapshots <= 0) return GNN_ERR_BAD_SIZE;
    for (int32_t t = 0; t < num_snapshots; ++t) out_graphs[t] = nullptr;
    if (!d_src || !d_dst || !num_edges) return GNN_ERR_NULL;
    if (num_nodes <= 0) return GNN_ERR_BAD_SIZE;
    for (int32_t t = 0; t < num_snapshots; ++t) {
        if (num_edges[t] < 0 || num_edges[t] >= (1ll << 31)) return GNN_ERR_BAD_SIZE;
        if (num_edges[t] > 0 && (!d_src[t] || !d_dst[t])) return GNN_ERR_NULL;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    int dev = 0;
    GNN_HIP(hipGetDevice(&dev));

    // one allocation for all graphs.  The temporaries come from the buffer the library keeps between builds: a flag
    // block per snapshot in front, then the job tables, then every snapshot's own sort buffers and counts (all
    // snapshots are built by the same launches: blockIdx.y names the snapshot).  One node (nothing to sort) takes
    // the builds one after the other with one set of temporaries.
    const bool one_by_one = num_nodes == 1;
    std::vector<gnn_graph *> graphs((size_t)num_snapshots, nullptr);
    std::vector<graph_layout> layouts((size_t)num_snapshots);
    std::vector<temp_layout> temps((size_t)num_snapshots);
    std::vector<size_t> base((size_t)num_snapshots), temp_base((size_t)num_snapshots);
    size_t slab_bytes = 0, temp_bytes = 0;
    int64_t max_edges = 0;
    const size_t flag_block = kFlagInts * sizeof(int32_t), flag_bytes = flag_block * (size_t)num_snapshots;
    const size_t jobs_bytes = (sizeof(BuildJob) * (size_t)num_snapshots + 255) & ~(size_t)255;
    const size_t scans_bytes = (sizeof(gnn_scan_job) * (size_t)num_snapshots + 255) & ~(size_t)255;
    const size_t table_bytes = one_by_one ? 0 : jobs_bytes + 2 * scans_bytes;
    gnn_status st = GNN_OK;
    void *slab = nullptr, *tmp = nullptr;
    temp_lease lease;   // handed back when the function returns: every path has synchronised the stream by then
    shared_slab *shared = nullptr;
    std::vector<int32_t> h_flags((size_t)num_snapshots * kFlagInts, 0);
    auto fail = [&](gnn_status code) {
        (void)hipStreamSynchronize(s);
        for (gnn_graph *g : graphs) delete g;
        if (slab) (void)hipFree(slab);
        delete shared;
        return code;
    };
    for (int32_t t = 0; t < num_snapshots; ++t) {
        gnn_graph *g = new (std::nothrow) gnn_graph();
        if (!g) return fail(GNN_ERR_ALLOC);
        graphs[(size_t)t] = g;
        int32_t small_max = 0, chunk = 0;
        (void)resolve_thresholds(num_edges[t], &small_max, &chunk);
        g->num_nodes = num_nodes;
        g->num_src_nodes = num_nodes;
        g->num_edges = num_edges[t];
        g->small_max = small_max;
        g->chunk = chunk;
        g->device = dev;
        layouts[(size_t)t] = plan_graph(num_edges[t], num_nodes, chunk);
        temps[(size_t)t] = plan_temp(num_edges[t], num_nodes);
        base[(size_t)t] = slab_bytes;
        slab_bytes += layouts[(size_t)t].bytes;
        temp_base[(size_t)t] = one_by_one ? 0 : temp_bytes;
        temp_bytes = one_by_one ? std::max(temp_bytes, temps[(size_t)t].bytes) : temp_bytes + temps[(size_t)t].bytes;
        max_edges = std::max(max_edges, num_edges[t]);
    }
    shared = new (std::nothrow) shared_slab();
    if (!shared) return fail(GNN_ERR_ALLOC);
    // like a single build, a batch takes over the arrays of a destroyed graph (or batch) of a similar size
    shared->device = dev;
    shared->bytes = slab_bytes ? slab_bytes : 256;
    if (!slab_cache_take(slab_bytes, dev, &slab, &shared->bytes) && (st = slab_alloc(&slab, slab_bytes)) != GNN_OK)
        return fail(st);
    if ((st = temp_acquire(&lease, flag_bytes + table_bytes + temp_bytes)) != GNN_OK) return fail(st);
    tmp = lease.ptr;
    if (hipMemsetAsync(tmp, 0, flag_bytes, s) != hipSuccess) return fail(GNN_ERR_DEVICE);
    char *tables = static_cast<char *>(tmp) + flag_bytes, *temp0 = tables + table_bytes;
    std::vector<char> h_tables(table_bytes);
    for (int32_t t = 0; t < num_snapshots; ++t) {
        gnn_graph *g = graphs[(size_t)t];
        bind_graph(g, static_cast<char *>(slab) + base[(size_t)t], layouts[(size_t)t]);
        int32_t *d_flag = reinterpret_cast<int32_t *>(static_cast<char *>(tmp) + flag_block * (size_t)t);
        char *ts = temp0 + temp_base[(size_t)t];
        const temp_layout &T = temps[(size_t)t];
        if (one_by_one) {
            st = enqueue_build(d_src[t], d_dst[t], num_edges[t], num_nodes, s, g, ts, T, d_flag);
            if (st != GNN_OK) return fail(st);
            continue;
        }
        if (num_edges[t] == 0 &&
            hipMemsetAsync(g->rowptr, 0, ((size_t)num_nodes + 1) * sizeof(int32_t), s) != hipSuccess)
            return fail(GNN_ERR_DEVICE);
        BuildJob j{};
        j.src = d_src[t]; j.dst = d_dst[t]; j.E = num_edges[t];
        j.num_tiles = (int32_t)T.num_tiles; j.small_max = g->small_max; j.chunk = g->chunk;
        j.kb = at(ts, T.o_kb); j.vb = at(ts, T.o_vb); j.eb = at(ts, T.o_eb); j.counts = at(ts, T.o_counts);
        j.digit_totals = at(ts, T.o_dtot); j.block_sums = at(ts, T.o_bsum); j.list_sizes = at(ts, T.o_sizes);
        j.flag = d_flag;
        j.rowptr = g->rowptr; j.indeg = g->indeg; j.colidx = g->colidx; j.perm = g->perm; j.rowidx = g->rowidx;
        j.dst_coo = g->dst_coo; j.dinv_loop = g->dinv_loop; j.dinv_plain = g->dinv_plain;
        j.small_rows = g->small_rows; j.item_row = g->item_row; j.item_start = g->item_start;
        j.item_slot = g->item_slot; j.split_rows = g->split_rows; j.split_slot0 = g->split_slot0;
        std::memcpy(h_tables.data() + sizeof(BuildJob) * (size_t)t, &j, sizeof(j));
        const gnn_scan_job counts_scan{j.counts, T.num_tiles, j.digit_totals};
        const gnn_scan_job lists_scan{j.block_sums, T.list_blocks, j.list_sizes};
        std::memcpy(h_tables.data() + jobs_bytes + sizeof(gnn_scan_job) * (size_t)t, &counts_scan, sizeof(counts_scan));
        std::memcpy(h_tables.data() + jobs_bytes + scans_bytes + sizeof(gnn_scan_job) * (size_t)t, &lists_scan,
                    sizeof(lists_scan));
    }
    if (!one_by_one) {
        if (hipMemcpyAsync(tables, h_tables.data(), table_bytes, hipMemcpyHostToDevice, s) != hipSuccess)
            return fail(GNN_ERR_DEVICE);
        st = enqueue_build_batch(reinterpret_cast<const BuildJob *>(tables),
                                 reinterpret_cast<const gnn_scan_job *>(tables + jobs_bytes),
                                 reinterpret_cast<const gnn_scan_job *>(tables + jobs_bytes + scans_bytes), num_snapshots,
                                 max_edges, num_nodes, s);
        if (st != GNN_OK) return fail(st);
    }
    if (hipMemcpyAsync(h_flags.data(), tmp, flag_bytes, hipMemcpyDeviceToHost, s) != hipSuccess) return fail(GNN_ERR_DEVICE);
    if (hipStreamSynchronize(s) != hipSuccess) return fail(GNN_ERR_DEVICE);
    for (int32_t t = 0; t < num_snapshots; ++t)
        if (h_flags[(size_t)t * kFlagInts + 8]) return fail(GNN_ERR_INDEX_RANGE);
    shared->ptr = slab;
    shared->refs.store(num_snapshots);
    for (int32_t t = 0; t < num_snapshots; ++t) {
        gnn_graph *g = graphs[(size_t)t];
        g->shared = shared;
        take_list_sizes(g, &h_flags[(size_t)t * kFlagInts + 8]);
        out_graphs[t] = g;
    }
    return GNN_OK;
}

int32_t gnn_graph_num_src_nodes(const gnn_graph *g) { return g ? g->num_src_nodes : 0; }

gnn_status gnn_release_cached_memory(void)
{
    {
        std::lock_guard<std::mutex> lock(g_slab_cache.mu);
        if (g_slab_cache.ptr) (void)hipFree(g_slab_cache.ptr);
        g_slab_cache.ptr = nullptr;
        g_slab_cache.bytes = 0;
        g_slab_cache.device = -1;
    }
    std::lock_guard<std::mutex> lock(g_temp_cache.mu);
    if (g_temp_cache.lent) return GNN_ERR_UNSUPPORTED;   // a build is running on another thread
    if (g_temp_cache.ptr) (void)hipFree(g_temp_cache.ptr);
    g_temp_cache.ptr = nullptr;
    g_temp_cache.bytes = 0;
    g_temp_cache.device = -1;
    return GNN_OK;
}

gnn_status gnn_graph_destroy(gnn_graph *g)
{
    if (!g) return GNN_OK;
    free_graph_arrays(g);
    delete g;
    return GNN_OK;
}

const int32_t *gnn_graph_rowptr(const gnn_graph *g) { return g ? g->rowptr : nullptr; }
const int32_t *gnn_graph_colidx(const gnn_graph *g) { return g ? g->colidx : nullptr; }
const int32_t *gnn_graph_perm(const gnn_graph *g) { return g ? g->perm : nullptr; }
const int32_t *gnn_graph_indegree(const gnn_graph *g) { return g ? g->indeg : nullptr; }
int32_t gnn_graph_num_nodes(const gnn_graph *g) { return g ? g->num_nodes : 0; }
int64_t gnn_graph_num_edges(const gnn_graph *g) { return g ? g->num_edges : 0; }

void gnn_graph_work_sizes(const gnn_graph *g, int32_t *n_small_rows, int32_t *n_items, int32_t *n_split_rows)
{
    if (n_small_rows) *n_small_rows = g ? g->n_small : 0;
    if (n_items) *n_items = g ? g->n_items : 0;
    if (n_split_rows) *n_split_rows = g ? g->n_split : 0;
}

void gnn_graph_work_lists(const gnn_graph *g, const int32_t **small_rows, const int32_t **item_row,
                          const int32_t **item_start, const int32_t **item_slot, const int32_t **split_rows,
                          const int32_t **split_slot0)
{
    if (small_rows) *small_rows = g ? g->small_rows : nullptr;
    if (item_row) *item_row = g ? g->item_row : nullptr;
    if (item_start) *item_start = g ? g->item_start : nullptr;
    if (item_slot) *item_slot = g ? g->item_slot : nullptr;
    if (split_rows) *split_rows = g ? g->split_rows : nullptr;
    if (split_slot0) *split_slot0 = g ? g->split_slot0 : nullptr;
}

gnn_status gnn_edge_data_to_csr(const gnn_graph *g, const float *d_e, int32_t e_dim, float *d_e_csr, void *stream)
{
    if (!g) return GNN_ERR_NULL;
    if (e_dim <= 0) return GNN_ERR_BAD_SIZE;
    if (g->num_edges == 0) return GNN_OK;
    if (!d_e || !d_e_csr) return GNN_ERR_NULL;
    if (e_dim == 1 && g->route && gnn_aligned16(d_e) && gnn_aligned16(d_e_csr))
        return gnn_route_coo_to_csr(g, d_e, d_e_csr, static_cast<hipStream_t>(stream));
    const int64_t total = g->num_edges * e_dim;
    const int blocks = (int)std::min<int64_t>(gnn_div_up(total, kThreads), 256 * 64);
    hipLaunchKernelGGL(permute_rows_kernel, dim3(blocks), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                       g->perm, g->num_edges, d_e, e_dim, d_e_csr);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

const char *gnn_status_string(gnn_status s)
{
    switch (s) {
    case GNN_OK: return "ok";
    case GNN_ERR_NULL: return "a required pointer is NULL";
    case GNN_ERR_BAD_SIZE: return "bad size, dimension or enum value";
    case GNN_ERR_INDEX_RANGE: return "node or graph index out of range";
    case GNN_ERR_UNSUPPORTED: return "combination not supported";
    case GNN_ERR_ALLOC: return "device allocation failed";
    case GNN_ERR_DEVICE: return "HIP call or kernel launch failed";
    case GNN_ERR_NOT_SORTED: return "graph_indicator is not sorted";
    case GNN_ERR_SCRATCH_LIMIT: return "the call needs more than the fixed scratch array of gnn_propagate_noalloc holds";
    case GNN_ERR_NOT_RESERVED: return "the graph's scratch memory is too small for this call: gnn_graph_reserve first";
    }
    return "unknown status";
}

}  // extern "C"

extern "C" gnn_status gnn_graph_reserve(gnn_graph *g, int32_t max_feat_dim, int32_t max_heads)
{
    if (!g) return GNN_ERR_NULL;
    if (max_feat_dim < 0 || max_heads < 0) return GNN_ERR_BAD_SIZE;
    const size_t need = gnn_scratch_floats(g->n_slots, g->num_nodes, max_feat_dim, max_heads);
    if (need <= g->scratch_floats) return GNN_OK;
    // Kernels enqueued earlier may still be using the buffer that is replaced.
    GNN_HIP(hipDeviceSynchronize());
    void *p = nullptr;
    if (hipMalloc(&p, need * sizeof(float)) != hipSuccess) {
        (void)hipGetLastError();
        return GNN_ERR_ALLOC;
    }
    if (g->own_scratch) (void)hipFree(g->own_scratch);
    g->own_scratch = p;
    g->scratch = static_cast<float *>(p);
    g->scratch_floats = need;
    return GNN_OK;
}
