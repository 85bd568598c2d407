// Two measurement aids: what the chip sustains, under its power limit, for the matrix
// instruction and for a streaming read.  A performance engineer reads a kernel's numbers
// against these as well as against the data-sheet peaks (PRAGMA, Section 3.2, lists matrix-unit
// activity and memory throughput among the evidence).  Not part of any operator.
//   * probe_mfma: every wave issues back-to-back matrix instructions on register operands
//     (the shapes the kernels use: 16 x 16 x 32 for bf16, 32 x 32 x 2 for fp32), independent
//     accumulators, two waves per SIMD -- nothing but the matrix pipe works.
//     With all-zero operands nothing toggles and the clock stays at its maximum; with random
//     operands the power limit lowers the clock, which is what a real GEMM sees.
//   * probe_mfma_fed: the same instruction with its operands re-read from LDS at the rate and
//     addresses of the large bf16 GEMM kernel, and optionally that kernel's global -> LDS copies:
//     what each kind of data movement costs in clock, with none of the GEMM's other work.
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
    f32x4 acc16[16];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc16[i] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
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
                // two 16 x 16 x 32 instructions (the shape the bf16 kernels use) per slot: the same
                // multiply-adds as one 32 x 32 x 16
                acc16[2 * q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[q % 4]),
                                                                       __builtin_bit_cast(bf16x8, wb[q / 4]), acc16[2 * q], 0, 0, 0);
                acc16[2 * q + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wa[(q + 1) % 4]),
                                                                           __builtin_bit_cast(bf16x8, wb[q / 4]), acc16[2 * q + 1], 0, 0, 0);
            } else {
                const unsigned int a = wa[q % 4][m / 8], b = wb[q / 4][m / 8];
                acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b),
                                                              acc[q], 0, 0, 0);
            }
        }
    }
    float t = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += acc[i][0] + acc[i][9] + acc16[2 * i][1] + acc16[2 * i + 1][2];
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

// The matrix instruction fed the way the large bf16 GEMM kernel feeds it, with nothing else of
// that kernel: 256 workgroups of eight waves (two per SIMD), each wave the 64 x 128 part of a
// 256 x 256 x 64 tile -- per "K tile" 64 instructions (16 x 16 x 32) whose operands it re-reads
// from LDS (per step of 32 along K four 128-bit reads for the A rows and sixteen transposing
// 64-bit reads for the B columns, at the kernel's swizzled addresses, in its order and in its
// sub-steps: 192 KiB per CU and tile), one barrier per tile, and with COPIES also the eight 1 KiB
// direct-to-LDS copies per wave and tile (64 KiB per CU) from `src`, issued in the tile's first
// sub-step and awaited before the barrier (two LDS stages: a copy has three quarters of a tile
// to land, less than in the kernel's deeper rings).
// The LDS holds small random bf16 values (then whatever the copies bring).  Tile t of workgroup w
// comes from the first `resident` 64 KiB pieces of src (w + t modulo resident: every piece is read
// by all workgroups, so it stays in L2) except every `stream_every`-th, which walks through the
// rest of src (a stream from memory).  Workgroup 0 reports the cycles and 100 MHz ticks of its loop.
template <bool COPIES>
__global__ __launch_bounds__(512) void probe_mfma_fed_kernel(int iters, const unsigned char* __restrict__ src,
                                                             unsigned int resident, unsigned int streamed,
                                                             int stream_every, unsigned long long* clock_out)
{
    constexpr int RA = 128, RB = 512, STAGE = 32768, TM = 4, TN = 8;
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a0[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a1[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_b0[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_b1[STAGE];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    {
        unsigned char* const all[4] = {lds_a0, lds_a1, lds_b0, lds_b1};
#pragma unroll
        for (int a = 0; a < 4; ++a)
            for (int c = tid; c < STAGE / 16; c += 512) {
                u32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    v[e] = (mix32((unsigned int)c * 747796405u + (a * 4 + e) * 2891336453u + blockIdx.x * 277803737u) & 0x807f807fu) | 0x3c003c00u;
                *(u32x4*)(all[a] + c * 16) = v;
            }
    }
    __syncthreads();

    // lane = (l16, grp): rows / columns l16 of a 16 x 16 block, k values 8 grp .. of a step of 32
    const int grp = lane >> 4, l16 = lane & 15;
    int a_koff[2], b_off[TN];
#pragma unroll
    for (int s = 0; s < 2; ++s) a_koff[s] = (wm * 64 + l16) * RA + (((4 * s + grp) ^ ((l16 / 2) % 8)) * 16);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = wn * 128 + 16 * j + 4 * (l16 & 3);
        const int krow = 8 * grp + (l16 >> 2);
        const int c = (n >> 3) ^ (4 * (krow & 3)) ^ (2 * ((krow >> 3) & 1));
        b_off[j] = krow * RB + c * 16 + (n & 7) * 2;
    }

    // sub-steps hs = 2 s + jh: the A fragments of step s (four, fetched with sub-step jh = 0) and
    // the B fragments j = 4 jh .. 4 jh + 3
    bf16x8 fa[2][TM];
    s16x4 fblo[2][4], fbhi[2][4];
    // fetch number q of what sub-step hs needs: A fragment 0, the eight halves of its B fragments,
    // the other A fragments (sub-steps with jh = 1: the B halves only)
    auto fetch_op = [&](const unsigned char* as, const unsigned char* bs, int hs, int q) __attribute__((always_inline)) {
        const int st = hs / 2, jh = hs % 2;
        const bool with_a = jh == 0;
        if (with_a && (q == 0 || q > 8)) {
            const int i = q == 0 ? 0 : q - 8;
            fa[st & 1][i] = *(const __attribute__((address_space(3))) bf16x8*)PGK_LDS(as + i * 16 * RA + a_koff[st]);
        } else {
            const int qb = with_a ? q - 1 : q;
            const int jj = qb / 2, h = qb % 2;
            const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)PGK_LDS(bs + b_off[4 * jh + jj] + (32 * st + 4 * h) * RB));
            if (h == 0) fblo[hs & 1][jj] = v; else fbhi[hs & 1][jj] = v;
        }
    };
    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    auto mfma_op = [&](int hs, int m) __attribute__((always_inline)) {
        const int st = hs / 2, jh = hs % 2;
        const int i = m / 4, jj = m % 4;
        const s16x8 both = __builtin_shufflevector(fblo[hs & 1][jj], fbhi[hs & 1][jj], 0, 1, 2, 3, 4, 5, 6, 7);
        acc[i][4 * jh + jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), fa[st & 1][i],
                                                                     acc[i][4 * jh + jj], 0, 0, 0);
    };
    // instruction m of this wave's share of the copy of one 64 KiB piece: 4 KiB of the A stage
    // (m < 4), 4 KiB of the B stage; every address stays inside the piece (the resource ends there)
    const unsigned int voff = (unsigned int)wave * 8192u + (unsigned int)lane * 16u;
    auto copy_op = [&](const unsigned char* piece, unsigned char* aw, unsigned char* bw, int m) __attribute__((always_inline)) {
        const auto rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)piece, 0, 65536, 0x00020000);
        unsigned char* dst = (m < 4 ? aw : bw) + wave * 4096 + (m % 4) * 1024;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, PGK_LDS(dst), 16, voff + (unsigned int)m * 1024u, 0, 0, 0);
    };
    // which piece the next tile copies: running indices, no division and no branch in the loop
    unsigned int r_idx = (unsigned int)blockIdx.x % resident;            // position in the resident pieces
    unsigned int s_idx = streamed ? (unsigned int)blockIdx.x % streamed : 0u;   // position in the streamed pieces
    const unsigned int s_step = streamed ? 256u % streamed : 0u;
    int until_stream = 0;                                                // tiles until the next streamed piece
    const bool streaming = stream_every > 0 && streamed > 0;
    auto next_piece = [&]() __attribute__((always_inline)) -> const unsigned char* {
        const bool from_stream = streaming && until_stream == 0;
        const unsigned int idx = from_stream ? resident + s_idx : r_idx;
        until_stream = from_stream ? stream_every - 1 : (streaming ? until_stream - 1 : 0);
        const unsigned int s_next = s_idx + s_step;
        s_idx = from_stream ? (s_next >= streamed ? s_next - streamed : s_next) : s_idx;
        const unsigned int r_next = r_idx + 1;
        r_idx = r_next == resident ? 0u : r_next;
        return src + (size_t)idx * 65536;
    };
    // One tile, in the GEMM kernel's order: operands from (ar, br); instruction m of a sub-step,
    // then the fetches of the next sub-step's operands that belong to slot m (spread over the
    // first twelve of the sixteen slots) and, in the first sub-step, a copy instruction of `piece`
    // into (aw, bw) -- the stages the previous tile was read from -- after every other slot.
    // Before the last sub-step's instructions: wait for the copies and this wave's LDS reads, meet
    // the other waves, and fetch the next tile's first operands from (aw, bw).  The order is
    // pinned by scheduling barriers, as in the kernel.
    auto tile = [&](const unsigned char* ar, const unsigned char* br, unsigned char* aw, unsigned char* bw,
                    const unsigned char* piece) __attribute__((always_inline)) {
#pragma unroll
        for (int hs = 0; hs < 4; ++hs) {
            const bool last = hs == 3;
            const int nhs = last ? 0 : hs + 1;                 // the sub-step whose operands are fetched now
            const int nq = nhs % 2 == 0 ? 12 : 8;
            if (last) {
                __builtin_amdgcn_sched_barrier(0);
                asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int m = 0; m < 16; ++m) {
                mfma_op(hs, m);
                __builtin_amdgcn_sched_barrier(0);
                const int q0 = m >= 12 ? nq : (m * nq) / 12, q1 = m + 1 >= 12 ? nq : ((m + 1) * nq) / 12;
#pragma unroll
                for (int q = q0; q < q1; ++q) fetch_op(last ? aw : ar, last ? bw : br, nhs, q);
                if constexpr (COPIES) {
                    if (hs == 0 && m % 2 == 0) copy_op(piece, aw, bw, m / 2);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

#pragma unroll
    for (int q = 0; q < 12; ++q) fetch_op(lds_a0, lds_b0, 0, q);
    const unsigned long long cyc0 = __builtin_readcyclecounter();
    const unsigned long long tick0 = __builtin_amdgcn_s_memrealtime();
    for (int t = 0; t < iters; t += 2) {          // iters is even (the launcher sees to it)
        tile(lds_a0, lds_b0, lds_a1, lds_b1, COPIES ? next_piece() : src);
        tile(lds_a1, lds_b1, lds_a0, lds_b0, COPIES ? next_piece() : src);
    }
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) sum += acc[i][j][0] + acc[i][j][3];
    const unsigned long long cyc1 = __builtin_readcyclecounter();
    const unsigned long long tick1 = __builtin_amdgcn_s_memrealtime();
    if (blockIdx.x == 0 && wave == 0) {
        clock_out[0] = cyc1 - cyc0;
        clock_out[1] = tick1 - tick0;
    }
    if (sum == 12345.678f) clock_out[2] = 1;      // keeps the work alive; never true in practice
}

}  // namespace

hipError_t launch_probe_mfma_fed(bool copies, int iters, const void* src, unsigned int resident, unsigned int streamed,
                                 int stream_every, unsigned long long* clock_out, hipStream_t s)
{
    if (iters < 2 || (iters & 1) || !clock_out) return hipErrorInvalidValue;
    if (copies && (!src || resident == 0)) return hipErrorInvalidValue;
    if (copies) hipLaunchKernelGGL(probe_mfma_fed_kernel<true>, dim3(256), dim3(512), 0, s, iters, (const unsigned char*)src, resident, streamed, stream_every, clock_out);
    else hipLaunchKernelGGL(probe_mfma_fed_kernel<false>, dim3(256), dim3(512), 0, s, iters, (const unsigned char*)src, 1u, 0u, 0, clock_out);
    return hipGetLastError();
}

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
