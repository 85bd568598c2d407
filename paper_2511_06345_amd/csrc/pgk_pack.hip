// Operand packing for GEMM shapes whose rows are not a whole number of 16-byte chunks
// (K or N not a multiple of 4 fp32 / 8 bf16 elements).  The matrix-core kernels copy operand
// tiles in 16-byte pieces, so such operands are first copied into buffers whose rows are padded
// with zeros to the next chunk (zeros add nothing to the products); an output whose rows would
// not even start on 4-byte boundaries (bf16, odd N) is computed one column wider and cropped.
// Streaming copies, a small fraction of the GEMM they make possible.
#include <hip/hip_runtime.h>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

namespace {

// dst[b][r][c] = src[b][r][c] for r < rows_src, c < cols_src, else 0; dst rows of cols_dst
// elements (a multiple of the chunk); one thread per 16-byte chunk of dst
template <typename T>
__global__ __launch_bounds__(256) void pad_matrix_kernel(const T* __restrict__ src, T* __restrict__ dst, long long batch,
                                                         int rows_src, int cols_src, int rows_dst, int cols_dst,
                                                         long long total_chunks)
{
    constexpr int EPC = 16 / (int)sizeof(T);
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total_chunks) return;
    const int cpr = cols_dst / EPC;
    const long long row = t / cpr;                     // b * rows_dst + r
    const int c0 = (int)(t - row * cpr) * EPC;
    const long long b = row / rows_dst;
    const int r = (int)(row - b * rows_dst);
    const T* s = src + ((size_t)b * (size_t)rows_src + (size_t)(r < rows_src ? r : 0)) * (size_t)cols_src;
    T v[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) v[e] = (r < rows_src && c0 + e < cols_src) ? s[c0 + e] : T(0);
    u32x4 out;
    __builtin_memcpy(&out, v, 16);
    *(u32x4*)(dst + (size_t)row * (size_t)cols_dst + c0) = out;
}

// dst[i] = i < n ? src[i] : 0 for i < n_dst
__global__ __launch_bounds__(256) void pad_vector_kernel(const float* __restrict__ src, float* __restrict__ dst, int n, int n_dst)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n_dst) dst[i] = (src && i < n) ? src[i] : 0.0f;
}

// dst[row][c] = src[row][c] for c < cols (dst rows of cols elements, src rows of cols_src)
template <typename T>
__global__ __launch_bounds__(256) void crop_matrix_kernel(const T* __restrict__ src, T* __restrict__ dst, long long rows,
                                                          int cols, int cols_src)
{
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= rows * cols) return;
    const long long row = t / cols;
    const int c = (int)(t - row * cols);
    dst[t] = src[(size_t)row * (size_t)cols_src + c];
}

}  // namespace

hipError_t launch_pad_matrix(const void* src, void* dst, long long batch, int rows_src, int cols_src, int rows_dst,
                             int cols_dst, int dtype, hipStream_t s)
{
    const int epc = dtype == DT_BF16 ? 8 : 4;
    if (cols_dst % epc != 0 || batch <= 0 || rows_dst < rows_src || cols_dst < cols_src) return hipErrorInvalidValue;
    const long long chunks = batch * rows_dst * (long long)(cols_dst / epc);
    const long long blocks = (chunks + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(pad_matrix_kernel<unsigned short>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned short*)src, (unsigned short*)dst, batch, rows_src, cols_src, rows_dst, cols_dst, chunks);
    else
        hipLaunchKernelGGL(pad_matrix_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s, (const float*)src, (float*)dst,
                           batch, rows_src, cols_src, rows_dst, cols_dst, chunks);
    return hipGetLastError();
}

hipError_t launch_pad_vector(const float* src, float* dst, int n, int n_dst, hipStream_t s)
{
    if (n_dst <= 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pad_vector_kernel, dim3((unsigned int)((n_dst + 255) / 256)), dim3(256), 0, s, src, dst, n, n_dst);
    return hipGetLastError();
}

hipError_t launch_crop_matrix(const void* src, void* dst, long long rows, int cols, int cols_src, int dtype, hipStream_t s)
{
    const long long blocks = (rows * cols + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL || cols_src < cols) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(crop_matrix_kernel<unsigned short>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned short*)src, (unsigned short*)dst, rows, cols, cols_src);
    else
        hipLaunchKernelGGL(crop_matrix_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s, (const float*)src, (float*)dst,
                           rows, cols, cols_src);
    return hipGetLastError();
}

}  // namespace pgk
