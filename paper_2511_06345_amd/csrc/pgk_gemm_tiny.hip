// Matrix-core GEMM + fused epilogue for latency-bound fp32 problems: a handful of output tiles
// and a K of a few hundred (the 256 x 256 x 256 workload).  Same operator as the other kernels
// (C = act(A*B + bias), optional row sums; PRAGMA Sections 1 and 4.2 name it, the definition is
// the textbook one).
//
// On such a problem the tiled kernels are bound by one chain of dependent matrix instructions
// per wave -- K/2 of them, 64 cycles each -- on a few CUs, while the rest of the chip idles.  Here
// the chain is cut four ways and spread over four times as many CUs:
//  * a workgroup owns a 32 x 32 tile of C; its four waves (one per SIMD) each take a contiguous
//    quarter of the K range and accumulate a partial 32 x 32 block with v_mfma_f32_32x32x2_f32;
//  * a wave stages its own slices of A and B (32 x 32 elements each per step of 32 along K)
//    through a private piece of LDS, two buffers deep, with 16-byte loads one step ahead; there
//    is no barrier in the main loop;
//  * the four partial blocks are added through LDS in wave order ((k0 + k1) + k2) + k3, then
//    bias, activation, 16-byte stores and the row sums, in a fixed order: equal inputs give
//    bit-equal outputs.
// Requirements (checked by the launcher): fp32, B as [K][ldb], K, N and ldb multiples of 4, A
// and B on 16-byte boundaries.  M and N need not be multiples of 32.
#include <hip/hip_runtime.h>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

namespace {

constexpr int TT = 32;          // tile edge
constexpr int TK = 32;          // K elements per staging step
constexpr int SA = 36;          // LDS row stride of the A slice in floats: 16 consecutive rows' 16-byte reads hit distinct banks
constexpr int SB = 40;          // ... of the B slice: rows 4 apart (the two half-waves) lie 32 banks apart
constexpr int WAVES = 4;

struct TinyStage {
    float a[TT * SA];           // [row][k]
    float b[TK * SB];           // [k][col]
};

}  // namespace

TileShape tiny_tile_shape() { return {TT, TT, TK}; }

__global__ __launch_bounds__(256) void gemm_tiny_f32_kernel(const GemmArgs p)
{
    __shared__ __attribute__((aligned(16))) TinyStage stage[WAVES][2];
    // the partial blocks of the four waves, [wave][row][col] (reuses nothing: 16 KiB)
    __shared__ __attribute__((aligned(16))) float part[WAVES][TT][TT + 4];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;

    const unsigned int tiles = (unsigned int)p.tiles_m * (unsigned int)p.tiles_n;
    const unsigned int b = blockIdx.x / tiles;
    const unsigned int r = blockIdx.x - b * tiles;
    const int tm = (int)(r / (unsigned int)p.tiles_n), tn = (int)(r - (unsigned int)tm * (unsigned int)p.tiles_n);
    const int m0 = tm * TT, n0 = tn * TT;

    // this wave's part of the K range: whole steps of TK, contiguous
    const int steps = (p.K + TK - 1) / TK;
    const int per = (steps + WAVES - 1) / WAVES;
    const int s_begin = wave * per;
    const int s_end = s_begin + per < steps ? s_begin + per : steps;

    const float* A = (const float*)p.A + (size_t)b * (size_t)p.a_batch_stride;
    const float* B = (const float*)p.B + (size_t)b * (size_t)p.b_batch_stride;

    // what this lane loads per step: four 16-byte chunks of the A slice (row ar[t], columns 4 ac[t] ..)
    // and four of the B slice (K row br[t], columns 4 bc[t] ..); chunk index = lane + 64 t
    f32x4 ra[4], rb[4];
    auto load_step = [&](int s) __attribute__((always_inline)) {
        const int k0 = s * TK;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int idx = lane + 64 * t;
            const int row = idx >> 3, c = idx & 7;
            const int gm = m0 + row, gk = k0 + 4 * c;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (gm < p.M && gk < p.K) v = *(const f32x4*)(A + (size_t)gm * (size_t)p.K + gk);
            ra[t] = v;
            const int gkr = k0 + row, gn = n0 + 4 * c;      // (same split of the index: K row, column chunk)
            f32x4 u = {0.f, 0.f, 0.f, 0.f};
            if (gkr < p.K && gn < p.N) u = *(const f32x4*)(B + (size_t)gkr * (size_t)p.ldb + gn);
            rb[t] = u;
        }
    };
    auto store_step = [&](TinyStage& st) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int idx = lane + 64 * t;
            const int row = idx >> 3, c = idx & 7;
            *(f32x4*)(st.a + row * SA + 4 * c) = ra[t];
            *(f32x4*)(st.b + row * SB + 4 * c) = rb[t];
        }
    };

    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    if (s_begin < s_end) load_step(s_begin);
    for (int s = s_begin; s < s_end; ++s) {
        TinyStage& st = stage[wave][(s - s_begin) & 1];
        store_step(st);
        if (s + 1 < s_end) load_step(s + 1);
        // the lanes of this wave read what other lanes of the same wave have just written: LDS
        // operations of one wave are carried out in order, the compiler must keep them so
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // four groups of eight K values: half-wave h multiplies k = 8 q + 4 h + e in instruction e
#pragma unroll
        for (int q = 0; q < TK / 8; ++q) {
            const f32x4 av = *(const f32x4*)(st.a + l32 * SA + 8 * q + 4 * half);
            float bv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) bv[e] = st.b[(8 * q + 4 * half + e) * SB + l32];
            // operand roles swapped as in the tiled kernels (B columns feed the first operand), so
            // that a lane's accumulators are one row of C in runs of four consecutive columns
#pragma unroll
            for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[e], av[e], acc, 0, 0, 0);
        }
        // (the buffer written two steps from now is this one: every lane is past its reads by then,
        // one wave executes its LDS operations in order)
        __builtin_amdgcn_wave_barrier();
    }

    // ---- the four partial blocks meet in LDS: lane (row l32, half h) holds columns 8 g + 4 h + e in acc[4 g + e]
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const f32x4 v = {acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
        *(f32x4*)(&part[wave][l32][8 * g + 4 * half]) = v;
    }
    __syncthreads();

    // ---- epilogue: thread t owns row t / 8, columns 4 (t % 8) .. + 3
    const int row = tid >> 3, c4 = (tid & 7) * 4;
    const int gm = m0 + row, gn = n0 + c4;
    f32x4 x = *(const f32x4*)(&part[0][row][c4]);
#pragma unroll
    for (int w = 1; w < WAVES; ++w) {
        const f32x4 y = *(const f32x4*)(&part[w][row][c4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] += y[e];
    }
    const bool live = gm < p.M && gn < p.N;      // N is a multiple of 4: a chunk is whole or absent
    float rs = 0.0f;
    if (live) {
        f32x4 bias = {0.f, 0.f, 0.f, 0.f};
        if (p.bias) {
#pragma unroll
            for (int e = 0; e < 4; ++e) bias[e] = p.bias[gn + e];
        }
        f32x4 y;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            y[e] = activate_dyn(x[e] + bias[e], p.act);
            rs += y[e];
        }
        typedef f32x4 f32x4_at_element __attribute__((aligned(4)));   // C may start on any element
        *(f32x4_at_element*)((float*)p.C + ((size_t)b * p.M + gm) * (size_t)p.N + gn) = y;
    }
    if (p.rs_part) {
        // the eight threads of a row are neighbours in a wave: fixed butterfly
        rs += __shfl_xor(rs, 1);
        rs += __shfl_xor(rs, 2);
        rs += __shfl_xor(rs, 4);
        if ((tid & 7) == 0 && gm < p.M)
            p.rs_part[((size_t)b * p.tiles_n + tn) * (size_t)p.M + gm] = rs;
    }
}

hipError_t launch_gemm_tiny(const GemmArgs& a, hipStream_t s)
{
    const long long wgs = (long long)a.tiles_m * a.tiles_n * a.batch;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.b_trans || a.bias_per_row || a.splits != 1 || a.k_rotate || a.conv_kw > 0) return hipErrorInvalidValue;
    if (a.K % 4 != 0 || a.N % 4 != 0 || a.ldb % 4 != 0) return hipErrorInvalidValue;
    if ((((uintptr_t)a.A) | ((uintptr_t)a.B)) % 16 != 0) return hipErrorInvalidValue;
    if ((a.a_batch_stride % 4) != 0 || (a.b_batch_stride % 4) != 0) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gemm_tiny_f32_kernel, dim3((unsigned int)wgs), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace pgk
