// Dense projection Z = X W on the matrix cores (fp32 MFMA, fp32 accumulate): the contraction
// inside GCNConv and the GAT layer (layers named in the paper, section 3).  X is tall and
// skinny ([rows x k], k ~ 100), W is small ([k x n], n <= a few hundred).
//
// A block of 4 wavefronts owns 128 rows x BN columns; each wavefront owns 32 rows and BN/32
// accumulator tiles of v_mfma_f32_32x32x2_f32.  W is staged through LDS in slabs of 64 k-values;
// X fragments go from global memory straight to registers: within a step of 8 k-values the
// lane (r = lane % 32, half = lane / 32) holds X[row0 + r][k0 + 4*half .. +3] and feeds value j of
// it to MFMA j, whose B operand is W[k0 + 4*half + j][col] -- the k order inside a step is
// permuted identically for both operands, which leaves the sum unchanged.
#include "gnn_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kRowsPerWave = 32;
constexpr int kRowsPerBlock = 4 * kRowsPerWave;
constexpr int kSlab = 64;   // k-values of W resident in LDS at a time

template <int NT /* 32-column tiles per block */, bool VEC4>
__global__ __launch_bounds__(kThreads) void xw_kernel(const float *__restrict__ x, int64_t rows, int k,
                                                      const float *__restrict__ w, int n,
                                                      const float *__restrict__ row_scale, float *__restrict__ z)
{
    constexpr int BN = NT * 32;
    __shared__ float ws[kSlab * BN];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, half = lane >> 5;
    const int64_t row0 = (int64_t)blockIdx.x * kRowsPerBlock + wave * kRowsPerWave;
    const int n0 = blockIdx.y * BN;
    const int64_t my_row = row0 + r;
    const bool row_ok = my_row < rows;
    const float *xrow = x + (row_ok ? my_row : 0) * (int64_t)k;

    floatx16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    for (int k0 = 0; k0 < k; k0 += kSlab) {
        __syncthreads();
        for (int idx = threadIdx.x; idx < kSlab * BN; idx += kThreads) {
            const int kk = idx / BN, c = idx - kk * BN;
            float v = 0.0f;
            if (k0 + kk < k && n0 + c < n) v = w[(int64_t)(k0 + kk) * n + n0 + c];
            ws[idx] = v;
        }
        __syncthreads();
        const int steps = (min(kSlab, k - k0) + 7) / 8;
        for (int s = 0; s < steps; ++s) {
            const int kb = k0 + s * 8 + half * 4;
            float a[4] = {0.f, 0.f, 0.f, 0.f};
            if (row_ok) {
                if constexpr (VEC4) {
                    if (kb < k) {   // k % 4 == 0: the four values are all inside the row
                        const float4 t = *reinterpret_cast<const float4 *>(xrow + kb);
                        a[0] = t.x; a[1] = t.y; a[2] = t.z; a[3] = t.w;
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (kb + j < k) a[j] = xrow[kb + j];
                }
            }
            const float *wrow = ws + (s * 8 + half * 4) * BN + r;
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[j], wrow[j * BN + t * 32], acc[t], 0, 0, 0);
        }
    }

    // Accumulator layout of the 32x32 tile: register v of lane l holds
    // row 8*(v/4) + 4*(l/32) + v%4, column l%32.
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int col = n0 + t * 32 + r;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t row = row0 + 8 * (v / 4) + 4 * half + (v % 4);
            if (row < rows && col < n) {
                float val = acc[t][v];
                if (row_scale) val *= row_scale[row];
                z[row * n + col] = val;
            }
        }
    }
}

}  // namespace

extern "C" gnn_status gnn_dense_xw(const float *d_x, int64_t rows, int32_t k, const float *d_w, int32_t n,
                                   const float *d_row_scale, float *d_z, void *stream)
{
    if (!d_x || !d_w || !d_z) return GNN_ERR_NULL;
    if (rows < 0 || k <= 0 || n <= 0) return GNN_ERR_BAD_SIZE;
    if (rows == 0) return GNN_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool vec4 = (k % 4 == 0) && ((reinterpret_cast<uintptr_t>(d_x) & 15u) == 0);
    const unsigned gx = (unsigned)gnn_div_up(rows, kRowsPerBlock);
    // Column tile: 128 wide when n is large enough, else the smallest multiple of 32 covering n.
    const int nt = n > 96 ? 4 : (n + 31) / 32;
    const unsigned gy = (unsigned)gnn_div_up(n, nt * 32);
    const dim3 grid(gx, gy), block(kThreads);
#define GNN_XW(NT)                                                                                              \
    do {                                                                                                        \
        if (vec4)                                                                                               \
            hipLaunchKernelGGL((xw_kernel<NT, true>), grid, block, 0, s, d_x, rows, k, d_w, n, d_row_scale, d_z);  \
        else                                                                                                    \
            hipLaunchKernelGGL((xw_kernel<NT, false>), grid, block, 0, s, d_x, rows, k, d_w, n, d_row_scale, d_z); \
    } while (0)
    switch (nt) {
    case 1: GNN_XW(1); break;
    case 2: GNN_XW(2); break;
    case 3: GNN_XW(3); break;
    default: GNN_XW(4); break;
    }
#undef GNN_XW
    GNN_LAUNCH_CHECK();
    return GNN_OK;
}
