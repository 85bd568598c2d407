// Fixed-order reductions that follow the GEMM kernels:
//  * rowsum_combine: adds the per-tile-column row-sum partials in tile order;
//  * splitk_reduce: second pass of the split-K path -- adds the K-slice partial
//    products in slice order, then bias, activation, store and row sum.
// No atomics: equal inputs give bit-equal outputs.  Both are streaming kernels
// bound by HBM bandwidth.
#include <hip/hip_runtime.h>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

__global__ __launch_bounds__(256) void rowsum_combine_kernel(const float* __restrict__ part,
                                                             float* __restrict__ rowsum,
                                                             int M, int batch, int tiles_n)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t total = (size_t)M * batch;
    if (i >= total) return;
    const size_t b = i / M, m = i - b * M;
    const float* src = part + b * (size_t)tiles_n * M + m;
    float s = src[0];
    for (int t = 1; t < tiles_n; ++t) s += src[(size_t)t * M];
    rowsum[i] = s;
}

hipError_t launch_rowsum_combine(const float* part, float* rowsum, int M, int batch, int tiles_n,
                                 hipStream_t s)
{
    const size_t total = (size_t)M * batch;
    const size_t blocks = (total + 255) / 256;
    if (blocks == 0 || blocks > 0x7fffffffULL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rowsum_combine_kernel, dim3((unsigned int)blocks), dim3(256), 0, s, part, rowsum, M,
                       batch, tiles_n);
    return hipGetLastError();
}

// One wave per output row and column segment (blockIdx.y; segments of seg_cols columns, so
// that skinny outputs still give enough waves).  VEC = 4 when N % 4 == 0 and the buffers are
// 16-byte aligned (each lane handles 4 consecutive columns per trip), else 1.  With several
// segments the row sums are per-segment partials rs_part[b][segment][m], to be added in
// segment order by rowsum_combine_kernel.
template <int VEC, bool OUT_BF16>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ ws,
                                                            const float* __restrict__ bias,
                                                            void* __restrict__ C, float* __restrict__ rowsum,
                                                            float* __restrict__ rs_part, int seg_cols,
                                                            int M, int N, int batch, int splits, int act)
{
    const int lane = threadIdx.x & 63;
    const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);   // b * M + m
    if (row >= (size_t)M * batch) return;
    const int seg = blockIdx.y, nseg = gridDim.y;
    const int n_begin = seg * seg_cols;
    const int n_end = n_begin + seg_cols < N ? n_begin + seg_cols : N;
    const size_t b = row / M, m = row - b * M;
    const size_t slice = (size_t)M * N;
    const float* src = ws + b * (size_t)splits * slice + m * (size_t)N;
    const size_t out = row * (size_t)N;

    float rs = 0.0f;
    for (int n = n_begin + lane * VEC; n < n_end; n += 64 * VEC) {
        float x[VEC];
        if constexpr (VEC == 4) {
            f32x4 v = *(const f32x4*)(src + n);
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = v[e];
            for (int s = 1; s < splits; ++s) {
                v = *(const f32x4*)(src + (size_t)s * slice + n);
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] += v[e];
            }
        } else {
            x[0] = src[n];
            for (int s = 1; s < splits; ++s) x[0] += src[(size_t)s * slice + n];
        }
        float y[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            y[e] = activate_dyn(x[e] + (bias ? bias[n + e] : 0.0f), act);
            rs += y[e];
        }
        if constexpr (VEC == 4) {
            if constexpr (OUT_BF16) {
                u32x2 pk = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                *(u32x2*)((unsigned short*)C + out + n) = pk;
            } else {
                f32x4 o = {y[0], y[1], y[2], y[3]};
                *(f32x4*)((float*)C + out + n) = o;
            }
        } else {
            if constexpr (OUT_BF16) ((unsigned short*)C)[out + n] = (unsigned short)(pack_bf16x2(y[0], 0.0f) & 0xffffu);
            else ((float*)C)[out + n] = y[0];
        }
    }
    if (rowsum) {
        // fixed butterfly over the 64 lanes
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) rs += __shfl_xor(rs, off);
        if (lane == 0) {
            if (nseg == 1) rowsum[row] = rs;
            else rs_part[(b * nseg + seg) * (size_t)M + m] = rs;
        }
    }
}

int splitk_reduce_segments(int M, int N, int batch)
{
    // about 4096 waves, segments of whole 256-column trips
    const long long rows = (long long)M * batch;
    long long want = (4096 + rows - 1) / rows;
    const long long most = (N + 255) / 256;
    if (want > most) want = most;
    if (want < 1) want = 1;
    const long long cols = (((N + want - 1) / want) + 255) / 256 * 256;
    return (int)((N + cols - 1) / cols);
}

hipError_t launch_splitk_reduce(const float* ws, const float* bias, void* C, float* rowsum, float* rs_part,
                                int nseg, int M, int N, int batch, int splits, int act, int dtype, hipStream_t s)
{
    const size_t rows = (size_t)M * batch;
    const size_t blocks = (rows + 3) / 4;
    if (blocks == 0 || blocks > 0x7fffffffULL || nseg < 1 || nseg > 65535) return hipErrorInvalidValue;
    const int seg_cols = (((N + nseg - 1) / nseg) + 255) / 256 * 256;
    const bool vec = (N % 4 == 0) && (((uintptr_t)ws | (uintptr_t)C | (uintptr_t)bias) % 16 == 0);
    const dim3 g((unsigned int)blocks, (unsigned int)nseg), t(256);
#define PGK_RED(V, BF) hipLaunchKernelGGL((splitk_reduce_kernel<V, BF>), g, t, 0, s, ws, bias, C, rowsum, rs_part, seg_cols, M, N, batch, splits, act)
    if (dtype == DT_BF16) { if (vec) PGK_RED(4, true); else PGK_RED(1, true); }
    else { if (vec) PGK_RED(4, false); else PGK_RED(1, false); }
#undef PGK_RED
    return hipGetLastError();
}

}  // namespace pgk
