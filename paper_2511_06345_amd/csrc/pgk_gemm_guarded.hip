// Bounds-checked GEMM + fused epilogue for shapes the matrix-core kernels do not
// take (sizes that are not tile multiples, unaligned pointers).  Same operator
// (C = act(A*B + bias), optional row sum; PRAGMA Sections 1 and 4.2 name it, the
// definition is the textbook one), same output modes, plain fp32 FMA arithmetic:
// a 64x64 tile per 256-thread workgroup, 4x4 outputs per thread, K in steps of 16
// through LDS.  Every global access is predicated on the matrix bounds.
#include <hip/hip_runtime.h>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

namespace {
constexpr int GT = 64;   // tile edge
constexpr int GK = 16;   // K step
}  // namespace

TileShape guarded_tile_shape() { return {GT, GT, GK}; }

template <bool BF16>
__device__ __forceinline__ float load_elem(const void* base, size_t idx)
{
    if constexpr (BF16) return bf16_bits_to_float(((const unsigned short*)base)[idx]);
    else return ((const float*)base)[idx];
}

template <bool BF16>
__global__ __launch_bounds__(256) void gemm_guarded_kernel(const GemmArgs p, const int out_mode)
{
    __shared__ float As[GK][GT + 4];   // [k][m]
    __shared__ float Bs[GK][GT + 4];   // [k][n]
    __shared__ float red[GT][17];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;

    const unsigned int tiles = (unsigned int)p.tiles_m * (unsigned int)p.tiles_n;
    const unsigned int z = blockIdx.x / tiles;
    const unsigned int r = blockIdx.x - z * tiles;
    const int tm = (int)(r / (unsigned int)p.tiles_n), tn = (int)(r - (unsigned int)tm * p.tiles_n);
    const int b = (int)(z / (unsigned int)p.splits);
    const int sp = (int)(z - (unsigned int)b * (unsigned int)p.splits);
    const int k_begin = sp * p.k_slice;
    const int k_end = (k_begin + p.k_slice < p.K) ? (k_begin + p.k_slice) : p.K;

    const int m0 = tm * GT, n0 = tn * GT;
    const size_t a_base = (size_t)b * (size_t)p.a_batch_stride;
    const size_t b_base = (size_t)b * (size_t)p.b_batch_stride;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;

    for (int k0 = k_begin; k0 < k_end; k0 += GK) {
        // A tile: 64 rows x 16 k, 4 elements per thread (k fastest in global memory)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;          // 0..1023
            const int mm = idx >> 4, kk = idx & 15;
            const int gm = m0 + mm, gk = k0 + kk;
            float v = 0.0f;
            if (gm < p.M && gk < k_end) v = load_elem<BF16>(p.A, a_base + (size_t)gm * p.K + gk);
            As[kk][mm] = v;
        }
        // B tile: 16 k x 64 cols (k fastest across threads when B is given transposed)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;
            const int kk = p.b_trans ? (idx & 15) : (idx >> 6), nn = p.b_trans ? (idx >> 4) : (idx & 63);
            const int gk = k0 + kk, gn = n0 + nn;
            float v = 0.0f;
            if (gk < k_end && gn < p.N) {
                if (p.conv_kw > 0) {
                    // convolution read in place: row gk is (input channel, tap), column gn an output position
                    const int ci = gk / p.conv_kw, tap = gk - ci * p.conv_kw;
                    const long long pos = (long long)gn * p.conv_stride + (long long)tap * p.conv_dil - p.conv_pad;
                    if (pos >= 0 && pos < p.conv_len)
                        v = load_elem<BF16>(p.B, b_base + (size_t)ci * (size_t)p.conv_len + (size_t)pos);
                } else if (p.b_trans) {
                    v = load_elem<BF16>(p.B, b_base + (size_t)gn * p.ldb + gk);
                } else {
                    v = load_elem<BF16>(p.B, b_base + (size_t)gk * p.ldb + gn);
                }
            }
            Bs[kk][nn] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            float a[4], bb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) bb[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], bb[j], acc[i][j]);
        }
        __syncthreads();
    }

    if (out_mode == 1) {
        float* w = p.ws + ((size_t)b * p.splits + sp) * (size_t)p.M * (size_t)p.N;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int gm = m0 + ty * 4 + i;
            if (gm >= p.M) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int gn = n0 + tx * 4 + j;
                if (gn < p.N) w[(size_t)gm * p.N + gn] = acc[i][j];
            }
        }
        return;
    }

    const size_t c_base = (size_t)b * p.M * p.N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int gm = m0 + ty * 4 + i;
        float rs = 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gn = n0 + tx * 4 + j;
            if (gm < p.M && gn < p.N) {
                const float x = acc[i][j] + (p.bias ? p.bias[p.bias_per_row ? gm : gn] : 0.0f);
                const float y = activate_dyn(x, p.act);
                rs += y;
                const size_t o = c_base + (size_t)gm * p.N + gn;
                if constexpr (BF16) ((unsigned short*)p.C)[o] = (unsigned short)(pack_bf16x2(y, 0.0f) & 0xffffu);
                else ((float*)p.C)[o] = y;
            }
        }
        red[ty * 4 + i][tx] = rs;
    }
    if (p.rs_part) {
        __syncthreads();
        if (tid < GT && m0 + tid < p.M) {
            float s = 0.0f;
#pragma unroll
            for (int t = 0; t < 16; ++t) s += red[tid][t];
            p.rs_part[((size_t)b * p.tiles_n + tn) * (size_t)p.M + (size_t)(m0 + tid)] = s;
        }
    }
}

hipError_t launch_gemm_guarded(const GemmArgs& a, int dtype, int out_mode, hipStream_t s)
{
    const long long wgs = (long long)a.tiles_m * a.tiles_n * a.batch * a.splits;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_BF16)
        hipLaunchKernelGGL(gemm_guarded_kernel<true>, dim3((unsigned int)wgs), dim3(256), 0, s, a, out_mode);
    else
        hipLaunchKernelGGL(gemm_guarded_kernel<false>, dim3((unsigned int)wgs), dim3(256), 0, s, a, out_mode);
    return hipGetLastError();
}

}  // namespace pgk
