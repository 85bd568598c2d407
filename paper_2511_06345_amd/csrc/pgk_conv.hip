// Helpers of the one-dimensional convolution (PRAGMA's second case study, Section 4.4
// "Conv Standard 1D"; the operator is the usual cross-correlation with zero padding).
// The convolution itself runs in the GEMM kernels: with stride 1,
//     y[b] (Cout x Lout) = sum over taps k of  W_k (Cout x Cin)  *  x[b] shifted by k * dilation - pad,
// so a K loop that walks tap after tap over the input channels reads, for each K tile, a plain
// sub-block of the padded input as its B operand.  What is needed beside that:
//   * conv_pad_input: the input with `pad` zeros in front of every row and zeros after it
//     up to a row length that keeps rows 16-byte aligned (skipped when there is no padding
//     and the rows are aligned already);
//   * conv_repack_weights: w[Cout][Cin][Kw] -> w'[Cout][Kw][Cin], so that the K index runs
//     over the channels inside a tap;
//   * conv_prepare: the regrouped weights together with the zero-padded strips that the tile
//     columns at the ends of the rows read when the input is used in place.
// All are streaming copies.
#include <hip/hip_runtime.h>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

namespace {

template <typename T>
__global__ __launch_bounds__(256) void conv_pad_input_kernel(const T* __restrict__ x, T* __restrict__ xp,
                                                             long long rows, int L, int Lp, int pad, long long second)
{
    // one workgroup row-slab: blockIdx.y = row (batch entry x channel), blockIdx.x = slab of 1024 outputs
    const long long row = blockIdx.y;
    if (row >= rows) return;
    const int j0 = blockIdx.x * 1024 + threadIdx.x;
    const T* src = x + (size_t)row * (size_t)L;
    T* dst = xp + (size_t)row * (size_t)Lp;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int j = j0 + 256 * u;
        if (j < Lp) {
            const int s = j - pad;
            dst[j] = (s >= 0 && s < L) ? src[s] : T(0);
            // the copy shifted left by one element, `second` elements further on
            if (second) dst[second + j] = (j + 1 < Lp && s + 1 >= 0 && s + 1 < L) ? src[s + 1] : T(0);
        }
    }
}

struct EdgeCols { int first[3]; };

template <typename T>
__global__ __launch_bounds__(256) void conv_repack_weights_kernel(const T* __restrict__ w, T* __restrict__ wr,
                                                                  int Cout, int Cin, int Kw, int even_first)
{
    const long long total = (long long)Cout * Cin * Kw;
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;     // index into wr: (co, slot, ci)
    if (t >= total) return;
    const int ci = (int)(t % Cin);
    const long long r = t / Cin;
    const int slot = (int)(r % Kw);
    const long long co = r / Kw;
    // which tap sits in this slot: in order, or the even taps followed by the odd ones
    const int n_even = (Kw + 1) / 2;
    const int k = !even_first ? slot : slot < n_even ? 2 * slot : 2 * (slot - n_even) + 1;
    wr[t] = w[(co * Cin + ci) * Kw + k];
}

// Both preparations of the in-place path in one launch (each is a few microseconds of work;
// a second launch costs as much again).  Workgroups [0, strip_blocks) fill the strips,
// strips[e][row][j] = x[row][first[e] + j] inside [0, L), else 0, numbered as (slab of 256
// columns, row, edge) with the slab fastest; the rest regroup the weights.
template <typename T>
__global__ __launch_bounds__(256) void conv_prepare_kernel(const T* __restrict__ x, T* __restrict__ strips, long long rows,
                                                           int L, int W, int slabs, EdgeCols cols, unsigned int strip_blocks,
                                                           const T* __restrict__ w, T* __restrict__ wr, int Cout, int Cin, int Kw)
{
    if (blockIdx.x < strip_blocks) {
        const unsigned int slab = blockIdx.x % (unsigned int)slabs;
        const unsigned int r = blockIdx.x / (unsigned int)slabs;
        const long long row = (long long)(r % (unsigned long long)rows);
        const int e = (int)(r / (unsigned long long)rows);
        const int j = (int)slab * 256 + (int)threadIdx.x;
        if (j >= W) return;
        const long long s = (long long)cols.first[e] + j;
        strips[((size_t)e * (size_t)rows + (size_t)row) * (size_t)W + j] =
            (s >= 0 && s < L) ? x[(size_t)row * (size_t)L + (size_t)s] : T(0);
        return;
    }
    const long long total = (long long)Cout * Cin * Kw;
    const long long t = (long long)(blockIdx.x - strip_blocks) * 256 + threadIdx.x;     // index into wr: (co, k, ci)
    if (t >= total) return;
    const int ci = (int)(t % Cin);
    const long long q = t / Cin;
    const int k = (int)(q % Kw);
    const long long co = q / Kw;
    wr[t] = w[(co * Cin + ci) * Kw + k];
}

}  // namespace

hipError_t launch_conv_prepare(const void* x, void* strips, long long rows, int L, int W, int n_edges, const int* first_col,
                               const void* w, void* wr, int Cout, int Cin, int Kw, int dtype, hipStream_t s)
{
    if (rows <= 0 || n_edges < 0 || n_edges > 3) return hipErrorInvalidValue;
    EdgeCols cols{};
    for (int e = 0; e < n_edges; ++e) cols.first[e] = first_col[e];
    const int slabs = (W + 255) / 256;
    const long long strip_blocks = n_edges > 0 ? (long long)slabs * rows * n_edges : 0;
    const long long repack_blocks = ((long long)Cout * Cin * Kw + 255) / 256;
    const long long blocks = strip_blocks + repack_blocks;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(conv_prepare_kernel<unsigned short>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned short*)x, (unsigned short*)strips, rows, L, W, slabs > 0 ? slabs : 1, cols,
                           (unsigned int)strip_blocks, (const unsigned short*)w, (unsigned short*)wr, Cout, Cin, Kw);
    else
        hipLaunchKernelGGL(conv_prepare_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s, (const float*)x,
                           (float*)strips, rows, L, W, slabs > 0 ? slabs : 1, cols, (unsigned int)strip_blocks,
                           (const float*)w, (float*)wr, Cout, Cin, Kw);
    return hipGetLastError();
}

hipError_t launch_conv_pad_input(const void* x, void* xp, long long rows, int L, int Lp, int pad, int copies, int dtype, hipStream_t s)
{
    if (rows <= 0 || rows > 65535LL * 65535LL || copies < 1 || copies > 2) return hipErrorInvalidValue;
    const long long second = copies == 2 ? rows * (long long)Lp : 0;    // elements between the two copies
    // grid.y is limited to 65535: fold the rows when there are more
    const unsigned int slabs = (unsigned int)((Lp + 1023) / 1024);
    for (long long r0 = 0; r0 < rows; r0 += 65535) {
        const long long n = rows - r0 < 65535 ? rows - r0 : 65535;
        const dim3 grid(slabs, (unsigned int)n);
        if (dtype == DT_BF16)
            hipLaunchKernelGGL(conv_pad_input_kernel<unsigned short>, grid, dim3(256), 0, s,
                               (const unsigned short*)x + (size_t)r0 * L, (unsigned short*)xp + (size_t)r0 * Lp, n, L, Lp, pad, second);
        else
            hipLaunchKernelGGL(conv_pad_input_kernel<float>, grid, dim3(256), 0, s,
                               (const float*)x + (size_t)r0 * L, (float*)xp + (size_t)r0 * Lp, n, L, Lp, pad, second);
    }
    return hipGetLastError();
}

hipError_t launch_conv_repack_weights(const void* w, void* wr, int Cout, int Cin, int Kw, int even_taps_first, int dtype, hipStream_t s)
{
    const long long total = (long long)Cout * Cin * Kw;
    const long long blocks = (total + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(conv_repack_weights_kernel<unsigned short>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned short*)w, (unsigned short*)wr, Cout, Cin, Kw, even_taps_first);
    else
        hipLaunchKernelGGL(conv_repack_weights_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const float*)w, (float*)wr, Cout, Cin, Kw, even_taps_first);
    return hipGetLastError();
}

}  // namespace pgk
