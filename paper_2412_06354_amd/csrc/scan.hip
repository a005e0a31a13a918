// Exclusive prefix sum of int32 (the "degree prefix scan" that turns in-degrees into rowptr,
// also used for the radix sort's digit offsets and for compacting the work lists).
//
// Two levels: every block reduces its tile, one block scans the block sums, every block
// then scans its tile starting from its offset.  A tile is 256 threads x 8 values.  Up to 2048 tiles the
// middle step is folded into the last one (each block adds up the sums before it); one tile is one kernel.
// The radix sort's [digit][tile] counts are scanned row by row instead (one block per digit, one kernel); the
// scatter pass adds the digits' bases itself.
#include "gnn_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kItems = 8;
constexpr int kTile = kThreads * kItems;

__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int t = __shfl_up(v, off, 64);
        if (lane >= off) v += t;
    }
    return v;
}

// Exclusive scan of one value per thread across the block; *total receives the block sum.
__device__ __forceinline__ int block_exclusive_scan(int v, int *total)
{
    __shared__ int wave_sums[kThreads / 64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = wave_inclusive_scan(v);
    if (lane == 63) wave_sums[w] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kThreads / 64; ++i) {
        int s = wave_sums[i];
        if (i < w) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

__global__ __launch_bounds__(kThreads) void scan_reduce_kernel(const int32_t *__restrict__ in, int64_t n,
                                                               int32_t *__restrict__ block_sums)
{
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    int s = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i)
        if (base + i < n) s += in[base + i];
    int total;
    (void)block_exclusive_scan(s, &total);
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// One block scans m values in place (exclusive), tile after tile with a running carry.
__global__ __launch_bounds__(kThreads) void scan_single_block_kernel(int32_t *__restrict__ data, int64_t m)
{
    int carry = 0;
    for (int64_t tile = 0; tile < m; tile += kTile) {
        const int64_t base = tile + (int64_t)threadIdx.x * kItems;
        int v[kItems];
        int s = 0;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            v[i] = (base + i < m) ? data[base + i] : 0;
            s += v[i];
        }
        int total;
        int run = carry + block_exclusive_scan(s, &total);
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            if (base + i < m) data[base + i] = run;
            run += v[i];
        }
        carry += total;
    }
}

// OFFSETS: 0 = the tile starts at zero (a one-tile scan), 1 = block_offsets holds the scanned block sums,
// 2 = block_offsets holds the raw block sums and the block adds up those before its own (at most kTile of them:
// saves the single-block kernel in between).
template <int OFFSETS>
__global__ __launch_bounds__(kThreads) void scan_downsweep_kernel(const int32_t *in, int32_t *out, int64_t n,
                                                                  int64_t n_out,
                                                                  const int32_t *__restrict__ block_offsets)
{
    int offset = 0;
    if constexpr (OFFSETS == 1) offset = block_offsets[blockIdx.x];
    if constexpr (OFFSETS == 2) {
        int mine = 0;
        for (int i = threadIdx.x; i < (int)blockIdx.x; i += kThreads) mine += block_offsets[i];
        int ignored = block_exclusive_scan(mine, &offset);
        (void)ignored;
    }
    const int64_t base = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kItems;
    int v[kItems];
    int s = 0;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        v[i] = (base + i < n) ? in[base + i] : 0;
        s += v[i];
    }
    int total;
    int run = offset + block_exclusive_scan(s, &total);
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        if (base + i < n_out) out[base + i] = run;   // position n (if asked for) receives the grand total
        run += v[i];
    }
}

// Exclusive prefix sums along every row of a [rows x cols] array, in place, and the row totals: one block of
// kRowThreads threads per row, kItems consecutive values per thread, chunk after chunk with a running carry.
constexpr int kRowThreads = 1024;

__global__ __launch_bounds__(kRowThreads) void scan_rows_kernel(int32_t *__restrict__ data, int64_t cols,
                                                                int32_t *__restrict__ row_totals)
{
    __shared__ int wave_sums[kRowThreads / 64];
    int32_t *row = data + (int64_t)blockIdx.x * cols;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int carry = 0;
    for (int64_t chunk = 0; chunk < cols; chunk += (int64_t)kRowThreads * kItems) {
        const int64_t base = chunk + (int64_t)threadIdx.x * kItems;
        int v[kItems];
        int s = 0;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            v[i] = (base + i < cols) ? row[base + i] : 0;
            s += v[i];
        }
        const int inc = wave_inclusive_scan(s);
        if (lane == 63) wave_sums[w] = inc;
        __syncthreads();
        int before = 0, total = 0;
#pragma unroll
        for (int q = 0; q < kRowThreads / 64; ++q) {
            const int t = wave_sums[q];
            if (q < w) before += t;
            total += t;
        }
        __syncthreads();   // wave_sums is rewritten by the next chunk
        int run = carry + before + inc - s;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            if (base + i < cols) row[base + i] = run;
            run += v[i];
        }
        carry += total;
    }
    if (threadIdx.x == 0) row_totals[blockIdx.x] = carry;
}

}  // namespace

gnn_status gnn_scan_rows_exclusive_i32(int32_t *d_data, int rows, int64_t cols, int32_t *d_row_totals,
                                       hipStream_t stream)
{
    if (rows < 0 || cols < 0) return GNN_ERR_BAD_SIZE;
    if (rows == 0) return GNN_OK;
    hipLaunchKernelGGL(scan_rows_kernel, dim3((unsigned)rows), dim3(kRowThreads), 0, stream, d_data, cols,
                       d_row_totals);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}

size_t gnn_scan_tmp_elems(int64_t n)
{
    return (size_t)gnn_div_up(n + 1, kTile) + 1;
}

gnn_status gnn_scan_exclusive_i32(const int32_t *d_in, int32_t *d_out, int64_t n, bool append_total,
                                  int32_t *d_tmp, hipStream_t stream)
{
    if (n < 0) return GNN_ERR_BAD_SIZE;
    const int64_t n_out = n + (append_total ? 1 : 0);
    if (n_out == 0) return GNN_OK;
    const int64_t blocks = gnn_div_up(n_out, kTile);
    if (blocks == 1) {   // one tile: one kernel
        hipLaunchKernelGGL(scan_downsweep_kernel<0>, dim3(1), dim3(kThreads), 0, stream, d_in, d_out, n, n_out,
                           (const int32_t *)nullptr);
        GNN_LAUNCH_CHECK();
        return GNN_OK;
    }
    hipLaunchKernelGGL(scan_reduce_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, d_in, n, d_tmp);
    GNN_LAUNCH_CHECK();
    if (blocks <= kTile) {   // every block adds up the sums of the blocks before it: two kernels
        hipLaunchKernelGGL(scan_downsweep_kernel<2>, dim3((unsigned)blocks), dim3(kThreads), 0, stream, d_in, d_out, n,
                           n_out, d_tmp);
        GNN_LAUNCH_CHECK();
        return GNN_OK;
    }
    hipLaunchKernelGGL(scan_single_block_kernel, dim3(1), dim3(kThreads), 0, stream, d_tmp, blocks);
    GNN_LAUNCH_CHECK();
    hipLaunchKernelGGL(scan_downsweep_kernel<1>, dim3((unsigned)blocks), dim3(kThreads), 0, stream, d_in, d_out, n,
                       n_out, d_tmp);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}
