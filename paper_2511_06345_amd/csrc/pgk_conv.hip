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

// One 16-byte chunk of the regrouped weights: wr[co][k][ci0 .. ci0 + EPC) = w[co][ci][k] for ci < Cin,
// 0 for the padding channels up to Cin_pad (a multiple of the chunk).  c: chunk index (co, k, ci / EPC).
template <typename T>
__device__ __forceinline__ void repack_weight_chunk(long long c, const T* __restrict__ w, T* __restrict__ wr,
                                                    int Cout, int Cin, int Cin_pad, int Kw)
{
    constexpr int EPC = 16 / (int)sizeof(T);
    const int cpr = Cin_pad / EPC;
    if (c >= (long long)Cout * Kw * cpr) return;
    const int ci0 = (int)(c % cpr) * EPC;
    const long long q = c / cpr;
    const int k = (int)(q % Kw);
    const long long co = q / Kw;
    T v[EPC];
#pragma unroll
    for (int u = 0; u < EPC; ++u) v[u] = ci0 + u < Cin ? w[(co * Cin + ci0 + u) * Kw + k] : T(0);
    u32x4 out;
    __builtin_memcpy(&out, v, 16);
    *(u32x4*)(wr + (size_t)c * EPC) = out;
}

// xc[c][b][ci][j] = x[b][ci][(j + h) * stride + phase - pad] (inside [0, L), ci < Cin; else 0) with
// c = phase * shifts + h.  One thread per 16-byte chunk of the copies (rows of Lq elements, a
// multiple of the chunk): element loads, one 16-byte store.  Also regroups the weights (padded to
// Cin_pad channels) into wr.
template <typename T>
__global__ __launch_bounds__(256) void conv_phase_copies_kernel(const T* __restrict__ x, T* __restrict__ xc, long long B,
                                                                int Cin, int Cin_pad, int L, int Lq, int pad, int stride,
                                                                int shifts, long long total_chunks,
                                                                const T* __restrict__ w, T* __restrict__ wr, int Cout, int Kw)
{
    constexpr int EPC = 16 / (int)sizeof(T);
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    // the threads after the copies regroup the weights (same launch: a second one costs as much
    // as either piece of work)
    if (t >= total_chunks) { repack_weight_chunk<T>(t - total_chunks, w, wr, Cout, Cin, Cin_pad, Kw); return; }
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
// a second launch costs as much again).  One thread per 16-byte chunk of output: threads
// [0, strip_chunks) fill the strips, strips[e][row][j] = x[row][first[e] + j] inside [0, L), else
// 0 (W, the strip's row length, is a multiple of the chunk), numbered (chunk of the row, row,
// edge) with the chunk fastest; the rest regroup the weights, wr[co][k][ci] = w[co][ci][k], eight
// (bf16) or four (fp32) consecutive ci per thread (Cin is a multiple of the chunk on this path).
template <typename T>
__global__ __launch_bounds__(256) void conv_prepare_kernel(const T* __restrict__ x, T* __restrict__ strips, long long rows,
                                                           int L, int W, EdgeCols cols, long long strip_chunks,
                                                           const T* __restrict__ w, T* __restrict__ wr, int Cout, int Cin, int Kw)
{
    constexpr int EPC = 16 / (int)sizeof(T);
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    T v[EPC];
    T* dst;
    if (t < strip_chunks) {
        const int cpr = W / EPC;                              // chunks per strip row
        const long long r = t / cpr;
        const int j0 = (int)(t - r * cpr) * EPC;
        const long long row = r % rows;
        const int e = (int)(r / rows);
        const T* src = x + (size_t)row * (size_t)L;
        const long long s0 = (long long)cols.first[e] + j0;
#pragma unroll
        for (int u = 0; u < EPC; ++u) {
            const long long sidx = s0 + u;
            v[u] = (sidx >= 0 && sidx < L) ? src[sidx] : T(0);
        }
        dst = strips + ((size_t)e * (size_t)rows + (size_t)row) * (size_t)W + j0;
    } else {
        repack_weight_chunk<T>(t - strip_chunks, w, wr, Cout, Cin, Cin, Kw);
        return;
    }
    u32x4 out;
    __builtin_memcpy(&out, v, 16);
    *(u32x4*)dst = out;
}

}  // namespace

hipError_t launch_conv_prepare(const void* x, void* strips, long long rows, int L, int W, int n_edges, const int* first_col,
                               const void* w, void* wr, int Cout, int Cin, int Kw, int dtype, hipStream_t s)
{
    const int epc = dtype == DT_BF16 ? 8 : 4;
    if (rows <= 0 || n_edges < 0 || n_edges > 3) return hipErrorInvalidValue;
    // whole 16-byte chunks on both sides (the callers' plan guarantees it), 16-byte aligned buffers
    if (Cin % epc != 0 || (n_edges > 0 && W % epc != 0)) return hipErrorInvalidValue;
    if (((uintptr_t)strips | (uintptr_t)wr) % 16 != 0) return hipErrorInvalidValue;
    EdgeCols cols{};
    for (int e = 0; e < n_edges; ++e) cols.first[e] = first_col[e];
    const long long strip_chunks = n_edges > 0 ? (long long)(W / epc) * rows * n_edges : 0;
    const long long repack_chunks = (long long)Cout * Kw * (Cin / epc);
    const long long blocks = (strip_chunks + repack_chunks + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(conv_prepare_kernel<unsigned short>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned short*)x, (unsigned short*)strips, rows, L, W, cols, strip_chunks,
                           (const unsigned short*)w, (unsigned short*)wr, Cout, Cin, Kw);
    else
        hipLaunchKernelGGL(conv_prepare_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s, (const float*)x,
                           (float*)strips, rows, L, W, cols, strip_chunks, (const float*)w, (float*)wr, Cout, Cin, Kw);
    return hipGetLastError();
}

hipError_t launch_conv_phase_copies(const void* x, void* xc, long long B, int Cin, int Cin_pad, int L, int Lq, int pad,
                                    int stride, int shifts, const void* w, void* wr, int Cout, int Kw, int dtype, hipStream_t s)
{
    const int epc = dtype == DT_BF16 ? 8 : 4;
    if (Lq % epc != 0 || Cin_pad % epc != 0 || B <= 0) return hipErrorInvalidValue;
    if (((uintptr_t)xc | (uintptr_t)wr) % 16 != 0) return hipErrorInvalidValue;
    const long long chunks = (long long)stride * shifts * B * Cin_pad * (Lq / epc);
    const long long repack_chunks = (long long)Cout * Kw * (Cin_pad / epc);
    const long long blocks = (chunks + repack_chunks + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(conv_phase_copies_kernel<unsigned short>, dim3((unsigned int)blocks), dim3(256), 0, s,
                           (const unsigned short*)x, (unsigned short*)xc, B, Cin, Cin_pad, L, Lq, pad, stride, shifts, chunks,
                           (const unsigned short*)w, (unsigned short*)wr, Cout, Kw);
    else
        hipLaunchKernelGGL(conv_phase_copies_kernel<float>, dim3((unsigned int)blocks), dim3(256), 0, s, (const float*)x,
                           (float*)xc, B, Cin, Cin_pad, L, Lq, pad, stride, shifts, chunks, (const float*)w, (float*)wr, Cout, Kw);
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
