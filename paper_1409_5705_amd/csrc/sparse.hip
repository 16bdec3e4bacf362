// Sparse (CSR) samples and second factors: validation and conversion into the
// dense, tile-aligned operand layouts the MFMA contractions read.
//
// At the densities of the workloads this library is sized for (about 10 % of
// the features non-zero, hundreds to thousands of factor pairs per step) every
// 32-wide block of every operand tile holds non-zeros, so the contraction itself
// stays a dense MFMA product; what sparsity saves is the interchange format (the
// bytes a factor block occupies and a peer would send) and the dense staging
// copies of X and V, which are written here directly in the layout the kernels
// consume.
#include "kernels.h"

namespace sfb {
namespace {

__device__ __forceinline__ uint16_t f32_to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);                                              // round to nearest even
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// One wavefront per CSR row: dst[r * row_stride + c * col_stride] = value (times
// coef[r] if given).  Entries whose column is outside [0, cols) and row ranges
// outside [0, nnz] are skipped, so malformed input cannot write out of bounds.
template <typename T>
__global__ __launch_bounds__(256) void csr_scatter_kernel(const int64_t* __restrict__ indptr,
                                                          const int32_t* __restrict__ indices,
                                                          const T* __restrict__ values,
                                                          const float* __restrict__ coef, T* __restrict__ dst,
                                                          int64_t rows, int64_t cols, int64_t nnz,
                                                          int64_t row_stride, int64_t col_stride)
{
    const int lane = threadIdx.x & 63;
    const int64_t waves = (int64_t)gridDim.x * 4;
    for (int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); r < rows; r += waves) {
        int64_t lo = indptr[r], hi = indptr[r + 1];
        if (lo < 0) lo = 0;
        if (hi > nnz) hi = nnz;
        const float c = coef ? coef[r] : 1.0f;
        for (int64_t t = lo + lane; t < hi; t += 64) {
            const int64_t col = indices[t];
            if (col < 0 || col >= cols) continue;
            T v = values[t];
            if (coef) {
                if constexpr (sizeof(T) == 2)
                    v = f32_to_bf16(c * bf16_to_f32(v));
                else
                    v = c * v;
            }
            // negative strides: blocks of 256 rows x 64 columns (the operand layout of the bf16 contractions);
            // col_stride = -pitch: the transpose, row_stride = -pitch: the matrix itself
            const int64_t at = col_stride < 0   ? ((col / 256) * (-col_stride / 64) + r / 64) * 16384 + (col % 256) * 64 + r % 64
                               : row_stride < 0 ? ((r / 256) * (-row_stride / 64) + col / 64) * 16384 + (r % 256) * 64 + col % 64
                                                : r * row_stride + col * col_stride;
            dst[at] = v;
        }
    }
}

// Counts violations of the format: indptr[0] == 0, indptr non-decreasing,
// indptr[rows] == nnz, column indices in [0, cols) and strictly increasing
// within a row.
__global__ __launch_bounds__(256) void csr_check_kernel(const int64_t* __restrict__ indptr,
                                                        const int32_t* __restrict__ indices, int64_t rows,
                                                        int64_t cols, int64_t nnz, unsigned int* __restrict__ bad)
{
    const int lane = threadIdx.x & 63;
    const int64_t waves = (int64_t)gridDim.x * 4;
    unsigned int mine = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (indptr[0] != 0) ++mine;
        if (indptr[rows] != nnz) ++mine;
    }
    for (int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); r < rows; r += waves) {
        const int64_t lo = indptr[r], hi = indptr[r + 1];
        if (lo < 0 || hi < lo || hi > nnz) {
            if (lane == 0) ++mine;
            continue;
        }
        for (int64_t t = lo + lane; t < hi; t += 64) {
            const int64_t col = indices[t];
            if (col < 0 || col >= cols) ++mine;
            else if (t > lo && (int64_t)indices[t - 1] >= col) ++mine;
        }
    }
    if (mine) atomicAdd(bad, mine);
}

unsigned wave_grid(int64_t rows)
{
    int64_t g = (rows + 3) / 4;
    if (g > 65536) g = 65536;
    return (unsigned)(g < 1 ? 1 : g);
}

}  // namespace

hipError_t launch_csr_scatter(const int64_t* indptr, const int32_t* indices, const void* values, bool bf16,
                              const float* coef, void* dst, int64_t rows, int64_t cols, int64_t nnz,
                              int64_t row_stride, int64_t col_stride, hipStream_t stream)
{
    if (rows <= 0 || nnz <= 0) return hipSuccess;
    if (bf16)
        hipLaunchKernelGGL((csr_scatter_kernel<uint16_t>), dim3(wave_grid(rows)), dim3(256), 0, stream, indptr, indices,
                           static_cast<const uint16_t*>(values), coef, static_cast<uint16_t*>(dst), rows, cols, nnz,
                           row_stride, col_stride);
    else
        hipLaunchKernelGGL((csr_scatter_kernel<float>), dim3(wave_grid(rows)), dim3(256), 0, stream, indptr, indices,
                           static_cast<const float*>(values), coef, static_cast<float*>(dst), rows, cols, nnz,
                           row_stride, col_stride);
    return hipGetLastError();
}

hipError_t launch_csr_check(const int64_t* indptr, const int32_t* indices, int64_t rows, int64_t cols, int64_t nnz,
                            unsigned int* bad, hipStream_t stream)
{
    hipLaunchKernelGGL(csr_check_kernel, dim3(wave_grid(rows)), dim3(256), 0, stream, indptr, indices, rows, cols, nnz,
                       bad);
    return hipGetLastError();
}

}  // namespace sfb
