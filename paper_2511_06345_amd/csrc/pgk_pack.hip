// Operand packing for GEMM shapes whose operand rows are not a whole number of 16-byte chunks
// (K, or the N of a plain B, not a multiple of 4 fp32 / 8 bf16 elements).  The matrix-core
// kernels copy operand tiles in 16-byte pieces, so such operands are first copied into buffers
// whose rows are padded with zeros to the next chunk (zeros add nothing to the products).
// A streaming copy, a small fraction of the GEMM it makes possible.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

namespace {

// dst[b][r][c] = src[b][r][c] for r < rows_src, c < cols_src, else 0; dst rows of cols_dst
// elements (a multiple of the chunk); one thread per 16-byte chunk of dst
template <typename T>
__global__ __launch_bounds__(256) void pad_matrix_kernel(const T* __restrict__ src, T* __restrict__ dst, int rows_src,
                                                         int cols_src, int rows_dst, int cols_dst, long long total_chunks)
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
    u32x4 out = {0u, 0u, 0u, 0u};
    if (r < rows_src) {
        if (c0 + EPC <= cols_src) {
            // a whole chunk of the source row: one 16-byte load from an element-aligned address
            using chunk_at_element = typename std::conditional<sizeof(T) == 2, u32x4_align2, u32x4_align4>::type;
            out = *(const chunk_at_element*)(s + c0);
        } else {
            T v[EPC];
#pragma unroll
            for (int e = 0; e < EPC; ++e) v[e] = c0 + e < cols_src ? s[c0 + e] : T(0);
            __builtin_memcpy(&out, v, 16);
        }
    }
    *(u32x4*)(dst + (size_t)row * (size_t)cols_dst + c0) = out;
}

// dst[b][n][k] = src[b][k][n] for k < K, 0 for K <= k < Kd (a B of few columns turned into its
// transposed form with rows of Kd elements, a multiple of the chunk); one thread per 16-byte
// chunk of dst.  The source is small (N is at most a tile's 32 columns), so its strided reads
// stay in the caches.
template <typename T>
__global__ __launch_bounds__(256) void transpose_pad_kernel(const T* __restrict__ src, T* __restrict__ dst, int K, int N,
                                                            int Kd, long long total_chunks)
{
    constexpr int EPC = 16 / (int)sizeof(T);
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total_chunks) return;
    const int cpr = Kd / EPC;
    const long long row = t / cpr;                     // b * N + n
    const int k0 = (int)(t - row * cpr) * EPC;
    const long long b = row / N;
    const int n = (int)(row - b * N);
    const T* s = src + (size_t)b * (size_t)K * (size_t)N + n;
    T v[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) v[e] = k0 + e < K ? s[(size_t)(k0 + e) * (size_t)N] : T(0);
    u32x4 out;
    __builtin_memcpy(&out, v, 16);
    *(u32x4*)(dst + (size_t)row * (size_t)Kd + k0) = out;
}

}  // namespace

hipError_t launch_transpose_pad(const void* src, void* dst, long long batch, int K, int N, int Kd, int dtype, hipStream_t s)
{
    const int epc = dtype == DT_BF16 ? 8 : 4;
    if (Kd % epc != 0 || batch <= 0 || Kd < K || N <= 0) return hipErrorInvalidValue;
    const long long chunks = batch * N * (long long)(Kd / epc);
    const long long blocks = (chunks + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(transpose_pad_kernel<unsigned short>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned short*)src, (unsigned short*)dst, K, N, Kd, chunks);
    else
        hipLaunchKernelGGL(transpose_pad_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s, (const float*)src,
                           (float*)dst, K, N, Kd, chunks);
    return hipGetLastError();
}

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
                           (const unsigned short*)src, (unsigned short*)dst, rows_src, cols_src, rows_dst, cols_dst, chunks);
    else
        hipLaunchKernelGGL(pad_matrix_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s, (const float*)src, (float*)dst,
                           rows_src, cols_src, rows_dst, cols_dst, chunks);
    return hipGetLastError();
}

}  // namespace pgk
