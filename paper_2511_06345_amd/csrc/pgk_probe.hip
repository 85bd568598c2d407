// Two measurement aids: what the chip sustains, under its power limit, for the matrix
// instruction and for a streaming read.  A performance engineer reads a kernel's numbers
// against these as well as against the data-sheet peaks (PRAGMA, Section 3.2, lists matrix-unit
// activity and memory throughput among the evidence).  Not part of any operator.
//   * probe_mfma: every wave issues back-to-back matrix instructions on register operands,
//     eight independent accumulators, two waves per SIMD -- nothing but the matrix pipe works.
//     With all-zero operands nothing toggles and the clock stays at its maximum; with random
//     operands the power limit lowers the clock, which is what a real GEMM sees.
//   * probe_stream_read: every lane reads 16 bytes at a time, grid-stride, and adds them up.
#include <hip/hip_runtime.h>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

namespace {

__device__ __forceinline__ unsigned int mix32(unsigned int h)
{
    h ^= h >> 15; h *= 0x2c1b3c6du; h ^= h >> 12; h *= 0x297a2d39u; h ^= h >> 15;
    return h;
}

template <bool BF16>
__global__ __launch_bounds__(256, 2) void probe_mfma_kernel(int iters, int random_operands, float* sink)
{
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
    u32x4 wa[4], wb[2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned int h = mix32(threadIdx.x * 747796405u + (i * 4 + e) * 2891336453u + blockIdx.x * 277803737u);
            // bf16 pairs (or one fp32) of magnitude about 0.01 with random sign and mantissa
            const unsigned int bits = BF16 ? ((h & 0x807f807fu) | 0x3c003c00u) : ((h & 0x807fffffu) | 0x3c000000u);
            wa[i][e] = random_operands ? bits : 0u;
            if (i < 2) wb[i][e] = random_operands ? (bits ^ (BF16 ? 0x00550033u : 0x00005533u)) : 0u;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int m = 0; m < 32; ++m) {
            const int q = m % 8;
            if constexpr (BF16) {
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wa[q % 4]),
                                                                 __builtin_bit_cast(bf16x8, wb[q / 4]), acc[q], 0, 0, 0);
            } else {
                const unsigned int a = wa[q % 4][m / 8], b = wb[q / 4][m / 8];
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b),
                                                              acc[q], 0, 0, 0);
            }
        }
    }
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += acc[i][0] + acc[i][9];
    if (t == 12345.678f) sink[0] = t;          // keeps the work alive; never true in practice
}

__global__ __launch_bounds__(256) void probe_stream_read_kernel(const u32x4* __restrict__ src, size_t chunks, float* sink)
{
    unsigned int s = 0;
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t step = (size_t)gridDim.x * 256;
    for (; c + 3 * step < chunks; c += stride) {
        const u32x4 a = __builtin_nontemporal_load(src + c), b = __builtin_nontemporal_load(src + c + step);
        const u32x4 d = __builtin_nontemporal_load(src + c + 2 * step), e = __builtin_nontemporal_load(src + c + 3 * step);
        s += a[0] ^ a[1] ^ a[2] ^ a[3] ^ b[0] ^ b[1] ^ b[2] ^ b[3] ^ d[0] ^ d[1] ^ d[2] ^ d[3] ^ e[0] ^ e[1] ^ e[2] ^ e[3];
    }
    for (; c < chunks; c += step) {
        const u32x4 a = __builtin_nontemporal_load(src + c);
        s += a[0] ^ a[1] ^ a[2] ^ a[3];
    }
    if (s == 0x12345679u) sink[0] = 1.0f;
}

}  // namespace

hipError_t launch_probe_mfma(int dtype, int random_operands, int iters, int workgroups, float* sink, hipStream_t s)
{
    if (dtype == DT_BF16) hipLaunchKernelGGL(probe_mfma_kernel<true>, dim3(workgroups), dim3(256), 0, s, iters, random_operands, sink);
    else hipLaunchKernelGGL(probe_mfma_kernel<false>, dim3(workgroups), dim3(256), 0, s, iters, random_operands, sink);
    return hipGetLastError();
}

hipError_t launch_probe_stream_read(const void* src, size_t bytes, float* sink, hipStream_t s)
{
    // two workgroups per CU, all sweeping the buffer together: 7.0 TB/s on a 2 GiB buffer; one per
    // CU gives 6.3, four 5.9, and one contiguous segment per workgroup 5.9 -- how much is in flight
    // decides, not contiguity
    hipLaunchKernelGGL(probe_stream_read_kernel, dim3(256 * 2), dim3(256), 0, s, (const u32x4*)src, bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace pgk
