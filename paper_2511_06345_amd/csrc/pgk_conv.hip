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
                                                             long long rows, int L, int Lp, int pad)
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
        }
    }
}

struct EdgeCols { int first[3]; };

template <typename T>
__global__ __launch_bounds__(256) void conv_repack_weights_kernel(const T* __restrict__ w, T* __restrict__ wr,
                                                                  int Cout, int Cin, int Cin_pad, int Kw)
{
    const long long total = (long long)Cout * Cin_pad * Kw;
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;     // index into wr: (co, k, ci)
    if (t >= total) return;
    const int ci = (int)(t % Cin_pad);
    const long long r = t / Cin_pad;
    const int k = (int)(r % Kw);
    const long long co = r / Kw;
    wr[t] = ci < Cin ? w[(co * Cin + ci) * Kw + k] : T(0);
}

// xc[c][b][ci][j] = x[b][ci][(j + h) * stride + phase - pad] (inside [0, L), ci < Cin; else 0) with
// c = phase * shifts + h.  One thread per 16-byte chunk of the copies (rows of Lq elements, a
// multiple of the chunk): element loads, one 16-byte store.
template <typename T>
__global__ __launch_bounds__(256) void conv_phase_copies_kernel(const T* __restrict__ x, T* __restrict__ xc, long long B,
                                                                int Cin, int Cin_pad, int L, int Lq, int pad, int stride,
                                                                int shifts, long long total_chunks)
{
    constexpr int EPC = 16 / (int)sizeof(T);
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= total_chunks) return;
    const int cpr = Lq / EPC;                                // chunks per row
    const long long row = t / cpr;                           // (c * B + b) * Cin_pad + ci
    const int j0 = (int)(t - row * cpr) * EPC;
    const int ci = (int)(row % Cin_pad);
    const long long cb = row / Cin_pad;
    const long long b = cb % B;
    const int c = (int)(cb / B);
    const int phase = c / shifts, h = c - phase * shifts;
    const T* src = x + ((size_t)b * (size_t)Cin + (size_t)(ci < Cin ? ci : 0)) * (size_t)L;
    T v[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
        const long long s = (long long)(j0 + e + h) * stride + phase - pad;
        v[e] = (ci < Cin && s >= 0 && s < L) ? src[s] : T(0);
    }
    u32x4 out;
    __builtin_memcpy(&out, v, 16);
    *(u32x4*)(xc + (size_t)row * (size_t)Lq + j0) = out;
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

hipError_t launch_conv_phase_copies(const void* x, void* xc, long long B, int Cin, int Cin_pad, int L, int Lq, int pad,
                                    int stride, int shifts, int dtype, hipStream_t s)
{
    const int epc = dtype == DT_BF16 ? 8 : 4;
    if (Lq % epc != 0 || B <= 0) return hipErrorInvalidValue;
    const long long chunks = (long long)stride * shifts * B * Cin_pad * (Lq / epc);
    const long long blocks = (chunks + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(conv_phase_copies_kernel<unsigned short>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned short*)x, (unsigned short*)xc, B, Cin, Cin_pad, L, Lq, pad, stride, shifts, chunks);
    else
        hipLaunchKernelGGL(conv_phase_copies_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s, (const float*)x,
                           (float*)xc, B, Cin, Cin_pad, L, Lq, pad, stride, shifts, chunks);
    return hipGetLastError();
}

hipError_t launch_conv_pad_input(const void* x, void* xp, long long rows, int L, int Lp, int pad, int dtype, hipStream_t s)
{
    if (rows <= 0 || rows > 65535LL * 65535LL) return hipErrorInvalidValue;
    // grid.y is limited to 65535: fold the rows when there are more
    const unsigned int slabs = (unsigned int)((Lp + 1023) / 1024);
    for (long long r0 = 0; r0 < rows; r0 += 65535) {
        const long long n = rows - r0 < 65535 ? rows - r0 : 65535;
        const dim3 grid(slabs, (unsigned int)n);
        if (dtype == DT_BF16)
            hipLaunchKernelGGL(conv_pad_input_kernel<unsigned short>, grid, dim3(256), 0, s,
                               (const unsigned short*)x + (size_t)r0 * L, (unsigned short*)xp + (size_t)r0 * Lp, n, L, Lp, pad);
        else
            hipLaunchKernelGGL(conv_pad_input_kernel<float>, grid, dim3(256), 0, s,
                               (const float*)x + (size_t)r0 * L, (float*)xp + (size_t)r0 * Lp, n, L, Lp, pad);
    }
    return hipGetLastError();
}

hipError_t launch_conv_repack_weights(const void* w, void* wr, int Cout, int Cin, int Cin_pad, int Kw, int dtype, hipStream_t s)
{
    const long long total = (long long)Cout * Cin_pad * Kw;
    const long long blocks = (total + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(conv_repack_weights_kernel<unsigned short>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned short*)w, (unsigned short*)wr, Cout, Cin, Cin_pad, Kw);
    else
        hipLaunchKernelGGL(conv_repack_weights_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const float*)w, (float*)wr, Cout, Cin, Cin_pad, Kw);
    return hipGetLastError();
}

}  // namespace pgk
