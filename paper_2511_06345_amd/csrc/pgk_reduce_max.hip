// Maximum over one dimension of a contiguous tensor viewed as [outer][red][inner]:
//     out[o][i] = max_r X[o][r][i],   idx[o][i] = smallest r attaining it
// (the reduction operator of PRAGMA's GPU case study, Section 4.4; the paper gives no
// formula, so this is the plain definition).  IEEE comparison: +0 and -0 tie and the
// earlier one is returned; a NaN in the slice gives that NaN and the first NaN's position.
//
// The kernels are streaming kernels bound by HBM bandwidth: every element is read once
// with 16-byte loads, several loads in flight per lane.
//   * inner == 1 (the reduced dimension is contiguous): a wave (short rows) or a
//     256-thread workgroup (long rows) sweeps one row in 16-byte chunks; lanes are
//     combined with cross-lane shuffles, waves through LDS.
//   * inner > 1: lanes lie along the contiguous inner dimension, 16 bytes each; the four
//     waves of a workgroup take every fourth r and are combined through LDS.
// Every combination step compares (value, position) pairs, so the result does not depend
// on how the work was split.  When there are too few outputs to fill the chip the reduced
// range is cut into segments (one workgroup each) and a second small kernel combines the
// segment results in order.
#include <hip/hip_runtime.h>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

namespace {

constexpr float kNegInf = -__builtin_huge_valf();
constexpr int kNoPos = 0x7fffffff;      // position of "no element seen"

// Does (xv at position xi) win over (mv at position mi)?  Positions differ unless both
// are kNoPos.  First NaN wins over everything; otherwise the larger value, and among
// equal values the earlier position.
__device__ __forceinline__ bool beats(float xv, int xi, float mv, int mi)
{
    const bool xn = xv != xv, mn = mv != mv;
    if (xn | mn) return xn && (!mn || xi < mi);
    return xv > mv || (xv == mv && xi < mi);
}

// The same for a scan in increasing position (xi > mi always): x replaces m when it is
// larger or the first NaN; an equal x never does.
__device__ __forceinline__ bool replaces(float xv, float mv) { return !(xv <= mv) && mv == mv; }

template <bool BF16>
struct Elem {
    static constexpr int BYTES = BF16 ? 2 : 4;
    static constexpr int VEC = 16 / BYTES;          // elements per 16-byte chunk
};

// widen the VEC elements of one 16-byte chunk to float (exact)
template <bool BF16>
__device__ __forceinline__ void unpack(const u32x4& w, float (&x)[Elem<BF16>::VEC])
{
    if constexpr (BF16) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned int lo = w[q] << 16, hi = w[q] & 0xffff0000u;
            x[2 * q] = __builtin_bit_cast(float, lo);
            x[2 * q + 1] = __builtin_bit_cast(float, hi);
        }
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned int bits = w[q];       // a value, not a vector-element lvalue, for the bit cast
            x[q] = __builtin_bit_cast(float, bits);
        }
    }
}

template <bool BF16>
__device__ __forceinline__ float load_one(const void* X, size_t e)
{
    if constexpr (BF16) return __builtin_bit_cast(float, (unsigned int)((const unsigned short*)X)[e] << 16);
    else return ((const float*)X)[e];
}

template <bool BF16>
__device__ __forceinline__ void store_one(void* out, size_t e, float v)
{
    if constexpr (BF16) ((unsigned short*)out)[e] = (unsigned short)(__builtin_bit_cast(unsigned int, v) >> 16);
    else ((float*)out)[e] = v;
}

// ---------------------------------------------------------------------------------
// inner == 1.  G lanes (one wave, or the whole workgroup of 256) sweep the chunks
// [c0, c1) of one row; lane l takes chunks c0 + l, c0 + l + G, ...  VEC == 1 is the
// fallback for rows that do not start on 16-byte boundaries (a "chunk" is one element).
// Result: direct to out / idx when segs == 1, else to the segment partials.
template <bool BF16, int VEC, int G>
__global__ __launch_bounds__(256) void reduce_max_rows_kernel(const void* __restrict__ X, void* __restrict__ out,
                                                              int* __restrict__ idx, float* __restrict__ pv,
                                                              int* __restrict__ pi, long long outer, int red,
                                                              int segs, int chunks_per_seg)
{
    constexpr int ROWS = 256 / G;                 // rows (or row segments) per workgroup
    constexpr int UNROLL = 4;
    __shared__ float sv[4];
    __shared__ int si[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int gl = tid % G;                       // lane within the group
    const long long unit = (long long)blockIdx.x * ROWS + tid / G;      // row * segs + seg
    const bool active = unit < outer * segs;      // whole groups only: uniform per wave
    const long long row = active ? unit / segs : 0;
    const int seg = active ? (int)(unit - row * segs) : 0;
    const int nch = red / VEC;
    const int c0 = seg * chunks_per_seg;
    const int c1 = active ? (c0 + chunks_per_seg < nch ? c0 + chunks_per_seg : nch) : c0;
    const size_t row_base = (size_t)row * (size_t)red;

    float bv[VEC];
    int bk[VEC];                                  // sweep number of the best element per slot
#pragma unroll
    for (int e = 0; e < VEC; ++e) { bv[e] = kNegInf; bk[e] = 0; }

    int c = c0 + gl, k = 0;
    if constexpr (VEC > 1) {
        const u32x4* src = (const u32x4*)((const unsigned char*)X + row_base * Elem<BF16>::BYTES);
        for (; c + (UNROLL - 1) * G < c1; c += UNROLL * G, k += UNROLL) {
            u32x4 w[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) w[u] = __builtin_nontemporal_load(src + c + u * G);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                float x[VEC];
                unpack<BF16>(w[u], x);
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    if (replaces(x[e], bv[e])) { bv[e] = x[e]; bk[e] = k + u; }
            }
        }
        for (; c < c1; c += G, ++k) {
            float x[VEC];
            unpack<BF16>(__builtin_nontemporal_load(src + c), x);
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                if (replaces(x[e], bv[e])) { bv[e] = x[e]; bk[e] = k; }
        }
    } else {
        for (; c < c1; c += G, ++k) {
            const float x = load_one<BF16>(X, row_base + c);
            if (replaces(x, bv[0])) { bv[0] = x; bk[0] = k; }
        }
    }
    // this lane's best: slot e of sweep k is element ((c0 + gl + k G) VEC + e) of the row
    const bool any = c0 + gl < c1;
    float v = kNegInf;
    int p = kNoPos;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const int pos = any ? (c0 + gl + bk[e] * G) * VEC + e : kNoPos;
        if (beats(bv[e], pos, v, p)) { v = bv[e]; p = pos; }
    }
    // across the lanes of the wave
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(v, off, 64);
        const int op = __shfl_xor(p, off, 64);
        if (beats(ov, op, v, p)) { v = ov; p = op; }
    }
    if constexpr (G == 256) {
        if (lane == 0) { sv[wave] = v; si[wave] = p; }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int w = 1; w < 4; ++w)
                if (beats(sv[w], si[w], v, p)) { v = sv[w]; p = si[w]; }
        }
    }
    if (gl == 0 && active) {
        if (segs == 1) {
            store_one<BF16>(out, (size_t)row, v);
            if (idx) idx[row] = p;
        } else {
            pv[unit] = v;
            pi[unit] = p;
        }
    }
}

// ---------------------------------------------------------------------------------
// inner > 1.  A workgroup owns 64 * VEC consecutive inner positions of one outer index
// and the r range of one segment; wave w takes r = r0 + w, r0 + w + 4, ...
template <bool BF16, int VEC>
__global__ __launch_bounds__(256) void reduce_max_cols_kernel(const void* __restrict__ X, void* __restrict__ out,
                                                              int* __restrict__ idx, float* __restrict__ pv,
                                                              int* __restrict__ pi, long long outer, int red,
                                                              long long inner, int tiles_i, int segs, int r_per_seg)
{
    // loads in flight per lane: four for fp32; two for bf16, whose eight slots per load keep the
    // vector ALU busier (measured on [32, 4096, 4096] bf16: 6000 GB/s with two, 5700 with four, 5350 with eight)
    constexpr int UNROLL = BF16 ? 2 : 4;
    __shared__ float sv[3][64 * VEC];
    __shared__ int si[3][64 * VEC];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    long long u = blockIdx.x;
    const int ti = (int)(u % tiles_i); u /= tiles_i;
    const int seg = (int)(u % segs);
    const long long o = u / segs;
    const long long i0 = (long long)ti * (64 * VEC) + (long long)lane * VEC;
    const bool in_range = i0 < inner;             // VEC > 1: inner is a multiple of VEC
    const int r0 = seg * r_per_seg;
    const int r1 = r0 + r_per_seg < red ? r0 + r_per_seg : red;

    float bv[VEC];
    int bp[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { bv[e] = kNegInf; bp[e] = kNoPos; }

    if (in_range) {
        const size_t base = ((size_t)o * (size_t)red) * (size_t)inner + (size_t)i0;   // element index of r = 0
        int r = r0 + wave;
        // the wave's first element starts the scan (so the loops need no "nothing seen yet" test)
        if constexpr (VEC > 1) {
            const unsigned char* src = (const unsigned char*)X + base * Elem<BF16>::BYTES;
            const size_t rstride = (size_t)inner * Elem<BF16>::BYTES;
            if (r < r1) {
                unpack<BF16>(__builtin_nontemporal_load((const u32x4*)(src + (size_t)r * rstride)), bv);
#pragma unroll
                for (int e = 0; e < VEC; ++e) bp[e] = r;
                r += 4;
            }
            for (; r + (UNROLL - 1) * 4 < r1; r += UNROLL * 4) {
                u32x4 w[UNROLL];
#pragma unroll
                for (int q = 0; q < UNROLL; ++q)
                    w[q] = __builtin_nontemporal_load((const u32x4*)(src + (size_t)(r + 4 * q) * rstride));
#pragma unroll
                for (int q = 0; q < UNROLL; ++q) {
                    float x[VEC];
                    unpack<BF16>(w[q], x);
#pragma unroll
                    for (int e = 0; e < VEC; ++e)
                        if (replaces(x[e], bv[e])) { bv[e] = x[e]; bp[e] = r + 4 * q; }
                }
            }
            for (; r < r1; r += 4) {
                float x[VEC];
                unpack<BF16>(__builtin_nontemporal_load((const u32x4*)(src + (size_t)r * rstride)), x);
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    if (replaces(x[e], bv[e])) { bv[e] = x[e]; bp[e] = r; }
            }
        } else {
            if (r < r1) { bv[0] = load_one<BF16>(X, base + (size_t)r * (size_t)inner); bp[0] = r; r += 4; }
            for (; r < r1; r += 4) {
                const float x = load_one<BF16>(X, base + (size_t)r * (size_t)inner);
                if (replaces(x, bv[0])) { bv[0] = x; bp[0] = r; }
            }
        }
    }
    // waves 1..3 hand their results to wave 0
    if (wave > 0) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { sv[wave - 1][lane * VEC + e] = bv[e]; si[wave - 1][lane * VEC + e] = bp[e]; }
    }
    __syncthreads();
    if (wave == 0 && in_range) {
#pragma unroll
        for (int w = 0; w < 3; ++w)
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float ov = sv[w][lane * VEC + e];
                const int op = si[w][lane * VEC + e];
                if (beats(ov, op, bv[e], bp[e])) { bv[e] = ov; bp[e] = op; }
            }
        const size_t dst = (size_t)o * (size_t)inner + (size_t)i0;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if (segs == 1) {
                store_one<BF16>(out, dst + e, bv[e]);
                if (idx) idx[dst + e] = bp[e];
            } else {
                const size_t at = ((size_t)o * segs + seg) * (size_t)inner + (size_t)i0 + e;
                pv[at] = bv[e];
                pi[at] = bp[e];
            }
        }
    }
}

// ---------------------------------------------------------------------------------
// inner == 1, short rows (at most 128 chunks): a wave per row would leave most lanes idle,
// so g = 1, 2, ... 32 lanes (a power of two, 1 << lg) share a row and a wave takes 64 / g
// rows; every lane has at most four chunks, fetched together.  No segments.
template <bool BF16, int VEC>
__global__ __launch_bounds__(256) void reduce_max_short_rows_kernel(const void* __restrict__ X, void* __restrict__ out,
                                                                    int* __restrict__ idx, long long outer, int red, int lg)
{
    const int tid = threadIdx.x;
    const int g = 1 << lg;
    const int gl = tid & (g - 1);
    const long long row = (long long)blockIdx.x * (256 >> lg) + (tid >> lg);
    const bool active = row < outer;              // whole groups only
    const int nch = red / VEC;
    const size_t row_base = (size_t)(active ? row : 0) * (size_t)red;

    float x[4][VEC];
    bool have[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int c = gl + u * g;
        have[u] = active && c < nch;
        if constexpr (VEC > 1) {
            u32x4 w = {0u, 0u, 0u, 0u};
            if (have[u]) w = __builtin_nontemporal_load((const u32x4*)((const unsigned char*)X + row_base * Elem<BF16>::BYTES) + c);
            unpack<BF16>(w, x[u]);
        } else {
            x[u][0] = have[u] ? load_one<BF16>(X, row_base + c) : 0.0f;
        }
    }
    // this lane's best over its chunks, in increasing position; the first one it has starts the scan
    float v = kNegInf;
    int p = kNoPos;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const int pos = (gl + u * g) * VEC + e;
            if (have[u] && (p == kNoPos || replaces(x[u][e], v))) { v = x[u][e]; p = pos; }
        }
    }
    // across the g lanes of the row
    for (int off = g >> 1; off > 0; off >>= 1) {
        const float ov = __shfl_xor(v, off, 64);
        const int op = __shfl_xor(p, off, 64);
        if (beats(ov, op, v, p)) { v = ov; p = op; }
    }
    if (gl == 0 && active) {
        store_one<BF16>(out, (size_t)row, v);
        if (idx) idx[row] = p;
    }
}

// ---------------------------------------------------------------------------------
// 1 < inner <= 64.  The strided kernel below would use inner / VEC of its 64 lanes.  Here
// one wave owns one outer index (and the r range of one segment) and sweeps that contiguous
// block of red x inner elements: R = 64 / inner consecutive r at a time, lane l at inner
// position l % inner of r number l / inner of the sweep -- 64 (or R * inner) consecutive
// elements per load instruction, eight sweeps in flight.  The lanes that share an inner
// position are then combined through LDS.
template <bool BF16>
__global__ __launch_bounds__(256) void reduce_max_small_inner_kernel(const void* __restrict__ X, void* __restrict__ out,
                                                                     int* __restrict__ idx, float* __restrict__ pv,
                                                                     int* __restrict__ pi, long long outer, int red,
                                                                     int inner, int segs, int r_per_seg)
{
    constexpr int UNROLL = 8;
    __shared__ float sv[4][64];
    __shared__ int si[4][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const long long unit = (long long)blockIdx.x * 4 + wave;        // o * segs + seg
    const bool active = unit < outer * segs;                        // uniform per wave
    const long long o = active ? unit / segs : 0;
    const int seg = active ? (int)(unit - o * segs) : 0;
    const int R = 64 / inner, L = R * inner;
    const int i = lane % inner, rr = lane / inner;
    const bool lane_ok = active && lane < L;
    const int r0 = seg * r_per_seg;
    const int r1 = active ? (r0 + r_per_seg < red ? r0 + r_per_seg : red) : r0;
    const size_t base = (size_t)o * (size_t)red * (size_t)inner + (size_t)i;

    float bv = kNegInf;
    int bp = kNoPos;
    int r = r0 + rr;
    if (lane_ok && r < r1) { bv = load_one<BF16>(X, base + (size_t)r * inner); bp = r; }   // starts the scan
    r += R;
    for (; r - rr + (UNROLL - 1) * R < r1; r += UNROLL * R) {       // uniform: all UNROLL sweeps start inside the range
        float x[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int ru = r + u * R;
            x[u] = (lane_ok && ru < r1) ? load_one<BF16>(X, base + (size_t)ru * inner) : kNegInf;
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
            if (lane_ok && r + u * R < r1 && replaces(x[u], bv)) { bv = x[u]; bp = r + u * R; }
    }
    for (; r - rr < r1; r += R) {
        if (lane_ok && r < r1) {
            const float x = load_one<BF16>(X, base + (size_t)r * inner);
            if (replaces(x, bv)) { bv = x; bp = r; }
        }
    }
    sv[wave][lane] = bv;
    si[wave][lane] = bp;
    __syncthreads();
    if (active && lane < inner) {
        float v = sv[wave][lane];
        int p = si[wave][lane];
        for (int q = 1; q < R; ++q) {
            const float ov = sv[wave][q * inner + lane];
            const int op = si[wave][q * inner + lane];
            if (beats(ov, op, v, p)) { v = ov; p = op; }
        }
        if (segs == 1) {
            store_one<BF16>(out, (size_t)o * inner + lane, v);
            if (idx) idx[(size_t)o * inner + lane] = p;
        } else {
            const size_t at = ((size_t)o * segs + seg) * (size_t)inner + lane;
            pv[at] = v;
            pi[at] = p;
        }
    }
}

// ---------------------------------------------------------------------------------
// inner > 1 and red x inner <= 128: the block of one outer index is smaller than a wave's
// worth of work.  A workgroup takes Q = 256 / (red x inner) outer indices: its threads load
// the Q blocks (contiguous in memory) into LDS, one element each, then one thread per output
// scans its red values in order.
template <bool BF16>
__global__ __launch_bounds__(256) void reduce_max_tiny_block_kernel(const void* __restrict__ X, void* __restrict__ out,
                                                                    int* __restrict__ idx, long long outer, int red, int inner)
{
    __shared__ float vals[256];
    const int tid = threadIdx.x;
    const int block = red * inner, Q = 256 / block;
    const long long o0 = (long long)blockIdx.x * Q;
    const int q_mine = tid / block;
    if (q_mine < Q && o0 + q_mine < outer) vals[tid] = load_one<BF16>(X, (size_t)o0 * (size_t)block + (size_t)tid);
    __syncthreads();
    const int q = tid / inner, i = tid - q * inner;
    if (q < Q && o0 + q < outer) {
        const float* mine = vals + q * block + i;
        float v = mine[0];
        int p = 0;
        for (int r = 1; r < red; ++r) {
            const float x = mine[r * inner];
            if (replaces(x, v)) { v = x; p = r; }
        }
        const size_t at = (size_t)(o0 + q) * (size_t)inner + (size_t)i;
        store_one<BF16>(out, at, v);
        if (idx) idx[at] = p;
    }
}

// Second pass: one thread per output, the segment results taken in order.
template <bool BF16>
__global__ __launch_bounds__(256) void reduce_max_finish_kernel(const float* __restrict__ pv, const int* __restrict__ pi,
                                                                void* __restrict__ out, int* __restrict__ idx,
                                                                long long outer, long long inner, int segs)
{
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= outer * inner) return;
    const long long o = t / inner, i = t - o * inner;
    const size_t base = (size_t)o * segs * (size_t)inner + (size_t)i;
    float v = pv[base];
    int p = pi[base];
    for (int s = 1; s < segs; ++s) {
        const float ov = pv[base + (size_t)s * (size_t)inner];
        const int op = pi[base + (size_t)s * (size_t)inner];
        if (beats(ov, op, v, p)) { v = ov; p = op; }
    }
    store_one<BF16>(out, (size_t)t, v);
    if (idx) idx[t] = p;
}

// The same with one wave per output, for many segments (few outputs, long rows): the lanes
// take every 64th segment, then the pairs are combined across the lanes.  The combine picks
// by (value, then earlier position), so the order it is applied in does not matter.
template <bool BF16>
__global__ __launch_bounds__(256) void reduce_max_finish_wave_kernel(const float* __restrict__ pv, const int* __restrict__ pi,
                                                                     void* __restrict__ out, int* __restrict__ idx,
                                                                     long long outer, long long inner, int segs)
{
    const int lane = threadIdx.x & 63;
    const long long t = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= outer * inner) return;          // whole waves leave together
    const long long o = t / inner, i = t - o * inner;
    const size_t base = (size_t)o * segs * (size_t)inner + (size_t)i;
    float v = kNegInf;
    int p = kNoPos;
    for (int s = lane; s < segs; s += 64) {
        const float ov = pv[base + (size_t)s * (size_t)inner];
        const int op = pi[base + (size_t)s * (size_t)inner];
        if (beats(ov, op, v, p)) { v = ov; p = op; }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(v, off, 64);
        const int op = __shfl_xor(p, off, 64);
        if (beats(ov, op, v, p)) { v = ov; p = op; }
    }
    if (lane == 0) {
        store_one<BF16>(out, (size_t)t, v);
        if (idx) idx[t] = p;
    }
}

// Workgroups a launch is cut into when the outputs alone give fewer: two per CU for fp32, four
// for bf16 (more vector ALU work per byte).  More, shorter segments stream worse -- measured on
// 1 GiB tensors, fp32 strided 6800 GB/s at 512 workgroups, 6500 at 1024, 6370 at 2048; bf16
// strided 5080 / 6450 / 5970; fp32 long rows 6940 / 6670 / 6620.
constexpr int target_workgroups(int dtype) { return dtype == DT_BF16 ? 1024 : 512; }
constexpr int kWaveFinishMinSegs = 16;
constexpr long long kShortRowChunks = 128;        // rows of at most this many chunks: several rows per wave
constexpr long long kSmallInner = 64;             // inner dimensions up to this: the flattened-sweep kernel
constexpr long long kTinyBlock = 128;             // red x inner up to this: several outer indices per workgroup

}  // namespace

ReducePlan plan_reduce_max(long long outer, long long red, long long inner, int dtype, bool x_aligned)
{
    ReducePlan pl{};
    const int es = dtype == DT_BF16 ? 2 : 4;
    const int vec16 = 16 / es;
    if (inner == 1) {
        pl.vec = (x_aligned && red % vec16 == 0) ? vec16 : 1;
        const long long nch = red / pl.vec;
        if (nch <= kShortRowChunks) {              // very short rows: g lanes each, at most four chunks per lane
            int g = 1;
            while (4 * g < nch) g *= 2;
            pl.group = g;
            pl.segs = 1;
            pl.per_seg = (int)nch;
            pl.tiles_i = 1;
            pl.blocks = (outer + 256 / g - 1) / (256 / g);
            pl.partial_elems = 0;
            return pl;
        }
        pl.group = nch <= 64 * 8 ? 64 : 256;       // short rows: one wave each
        pl.segs = 1;
        if (pl.group == 256 && outer < target_workgroups(dtype)) {
            const long long want = (target_workgroups(dtype) + outer - 1) / outer;
            const long long most = nch / (256 * 8) > 0 ? nch / (256 * 8) : 1;   // eight sweeps per segment at least
            pl.segs = (int)(want < most ? want : most);
        }
        pl.per_seg = (int)((nch + pl.segs - 1) / pl.segs);
        pl.segs = (int)((nch + pl.per_seg - 1) / pl.per_seg);
        const long long units = outer * pl.segs, per_wg = 256 / pl.group;
        pl.blocks = (units + per_wg - 1) / per_wg;
        pl.tiles_i = 1;
    } else if (red * inner <= kTinyBlock) {
        // several outer indices per workgroup; group = -1 marks this kernel
        pl.vec = 1;
        pl.group = -1;
        pl.tiles_i = 1;
        pl.segs = 1;
        pl.per_seg = (int)red;
        const long long q = 256 / (red * inner);
        pl.blocks = (outer + q - 1) / q;
    } else if (inner <= kSmallInner) {
        // one wave per (outer index, segment); group = 0 marks this kernel
        pl.vec = 1;
        pl.group = 0;
        pl.tiles_i = 1;
        pl.segs = 1;
        const long long waves = 4LL * target_workgroups(dtype);
        if (outer < waves) {
            const long long want = (waves + outer - 1) / outer;
            const long long sweep = 64 / inner;                                  // r per sweep
            const long long most = red / (8 * sweep) > 0 ? red / (8 * sweep) : 1;   // eight sweeps per segment at least
            pl.segs = (int)(want < most ? want : most);
        }
        pl.per_seg = (int)((red + pl.segs - 1) / pl.segs);
        pl.segs = (int)((red + pl.per_seg - 1) / pl.per_seg);
        pl.blocks = (outer * pl.segs + 3) / 4;
    } else {
        pl.vec = (x_aligned && inner % vec16 == 0) ? vec16 : 1;
        pl.group = 256;
        pl.tiles_i = (int)((inner + 64 * pl.vec - 1) / (64 * pl.vec));
        const long long wg0 = outer * pl.tiles_i;
        pl.segs = 1;
        if (wg0 < target_workgroups(dtype)) {
            const long long want = (target_workgroups(dtype) + wg0 - 1) / wg0;
            const long long most = red / 32 > 0 ? red / 32 : 1;                 // eight r per wave at least
            pl.segs = (int)(want < most ? want : most);
        }
        pl.per_seg = (int)((red + pl.segs - 1) / pl.segs);
        pl.segs = (int)((red + pl.per_seg - 1) / pl.per_seg);
        pl.blocks = wg0 * pl.segs;
    }
    pl.partial_elems = pl.segs > 1 ? (size_t)outer * pl.segs * (size_t)inner : 0;
    return pl;
}

hipError_t launch_reduce_max(const ReducePlan& pl, const void* X, void* out, int* idx, float* pv, int* pi,
                             long long outer, long long red, long long inner, int dtype, hipStream_t s)
{
    if (pl.blocks <= 0 || pl.blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned int)pl.blocks), block(256);
    const bool bf = dtype == DT_BF16;
    if (inner == 1 && pl.group < 64) {
        int lg = 0;
        while ((1 << lg) < pl.group) ++lg;
#define PGK_SHORT(BF, VEC) \
    hipLaunchKernelGGL((reduce_max_short_rows_kernel<BF, VEC>), grid, block, 0, s, X, out, idx, outer, (int)red, lg)
        if (bf) { if (pl.vec > 1) PGK_SHORT(true, 8); else PGK_SHORT(true, 1); }
        else { if (pl.vec > 1) PGK_SHORT(false, 4); else PGK_SHORT(false, 1); }
#undef PGK_SHORT
    } else if (inner > 1 && pl.group == -1) {
        if (bf) hipLaunchKernelGGL(reduce_max_tiny_block_kernel<true>, grid, block, 0, s, X, out, idx, outer, (int)red, (int)inner);
        else hipLaunchKernelGGL(reduce_max_tiny_block_kernel<false>, grid, block, 0, s, X, out, idx, outer, (int)red, (int)inner);
    } else if (inner > 1 && pl.group == 0) {
        if (bf) hipLaunchKernelGGL(reduce_max_small_inner_kernel<true>, grid, block, 0, s, X, out, idx, pv, pi, outer, (int)red, (int)inner, pl.segs, pl.per_seg);
        else hipLaunchKernelGGL(reduce_max_small_inner_kernel<false>, grid, block, 0, s, X, out, idx, pv, pi, outer, (int)red, (int)inner, pl.segs, pl.per_seg);
    } else if (inner == 1) {
#define PGK_ROWS(BF, VEC, G) \
    hipLaunchKernelGGL((reduce_max_rows_kernel<BF, VEC, G>), grid, block, 0, s, X, out, idx, pv, pi, outer, (int)red, pl.segs, pl.per_seg)
        if (bf) {
            if (pl.vec > 1) { if (pl.group == 64) PGK_ROWS(true, 8, 64); else PGK_ROWS(true, 8, 256); }
            else { if (pl.group == 64) PGK_ROWS(true, 1, 64); else PGK_ROWS(true, 1, 256); }
        } else {
            if (pl.vec > 1) { if (pl.group == 64) PGK_ROWS(false, 4, 64); else PGK_ROWS(false, 4, 256); }
            else { if (pl.group == 64) PGK_ROWS(false, 1, 64); else PGK_ROWS(false, 1, 256); }
        }
#undef PGK_ROWS
    } else {
#define PGK_COLS(BF, VEC) \
    hipLaunchKernelGGL((reduce_max_cols_kernel<BF, VEC>), grid, block, 0, s, X, out, idx, pv, pi, outer, (int)red, inner, pl.tiles_i, pl.segs, pl.per_seg)
        if (bf) { if (pl.vec > 1) PGK_COLS(true, 8); else PGK_COLS(true, 1); }
        else { if (pl.vec > 1) PGK_COLS(false, 4); else PGK_COLS(false, 1); }
#undef PGK_COLS
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.segs == 1) return e;
    const long long outs = outer * inner;
    if (pl.segs >= kWaveFinishMinSegs) {
        const long long wb = (outs + 3) / 4;
        if (wb > 0x7fffffffLL) return hipErrorInvalidValue;
        if (bf) hipLaunchKernelGGL(reduce_max_finish_wave_kernel<true>, dim3((unsigned int)wb), block, 0, s, pv, pi, out, idx, outer, inner, pl.segs);
        else hipLaunchKernelGGL(reduce_max_finish_wave_kernel<false>, dim3((unsigned int)wb), block, 0, s, pv, pi, out, idx, outer, inner, pl.segs);
        return hipGetLastError();
    }
    const long long fb = (outs + 255) / 256;
    if (fb > 0x7fffffffLL) return hipErrorInvalidValue;
    if (bf) hipLaunchKernelGGL(reduce_max_finish_kernel<true>, dim3((unsigned int)fb), block, 0, s, pv, pi, out, idx, outer, inner, pl.segs);
    else hipLaunchKernelGGL(reduce_max_finish_kernel<false>, dim3((unsigned int)fb), block, 0, s, pv, pi, out, idx, outer, inner, pl.segs);
    return hipGetLastError();
}

}  // namespace pgk
