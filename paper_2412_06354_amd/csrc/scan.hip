// Exclusive prefix sums of int32 along the rows of a small row-major array: the radix sort's [digit][tile] counts
// (one row per digit; the scatter pass adds the digits' bases itself) and the work lists' [list][block] counts.
// One block per row, eight consecutive values per thread, chunk after chunk with a running carry; the row totals
// are written next to the sums.
#include "gnn_internal.h"

namespace {

constexpr int kItems = 8;
constexpr int kRowThreads = 1024;

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

__device__ __forceinline__ void scan_row_body(int32_t *__restrict__ data, int64_t cols,
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

__global__ __launch_bounds__(kRowThreads) void scan_rows_kernel(int32_t *__restrict__ data, int64_t cols,
                                                                int32_t *__restrict__ row_totals)
{
    scan_row_body(data, cols, row_totals);
}

// One array per job: blockIdx.y names the job, blockIdx.x its row.
__global__ __launch_bounds__(kRowThreads) void scan_rows_jobs_kernel(const gnn_scan_job *__restrict__ jobs)
{
    const gnn_scan_job j = jobs[blockIdx.y];
    scan_row_body(j.data, j.cols, j.row_totals);
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

gnn_status gnn_scan_rows_exclusive_i32_jobs(const gnn_scan_job *d_jobs, int num_jobs, int rows, hipStream_t stream)
{
    if (rows < 0 || num_jobs < 0) return GNN_ERR_BAD_SIZE;
    if (rows == 0 || num_jobs == 0) return GNN_OK;
    hipLaunchKernelGGL(scan_rows_jobs_kernel, dim3((unsigned)rows, (unsigned)num_jobs), dim3(kRowThreads), 0, stream,
                       d_jobs);
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}
