// Device-side helpers shared by the HIP kernels: vector types, the fp32
// activation functions of the epilogue and bf16 packing.
#ifndef PGK_DEVICE_H
#define PGK_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pgk_kernels.h"

namespace pgk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// the same 16 bytes at an address that is only aligned to a 2- or 4-byte element (global memory
// takes multi-dword accesses at any alignment)
typedef u32x4 u32x4_align2 __attribute__((aligned(2)));
typedef u32x4 u32x4_align4 __attribute__((aligned(4)));

#define PGK_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define PGK_GLB(p) ((const __attribute__((address_space(1))) void*)(p))

// exp(z) through the hardware base-2 exponential.
__device__ __forceinline__ float fast_exp(float z)
{
    return __builtin_amdgcn_exp2f(z * 1.4426950408889634f);
}

// Logistic function times x, written so that no cancellation occurs:
// x * sigma(t) = x / (1 + exp(-t)).
__device__ __forceinline__ float x_sigmoid(float x, float t)
{
    return x * __builtin_amdgcn_rcpf(1.0f + fast_exp(-t));
}

// Epilogue activations in fp32.  The tanh form of GELU is evaluated as
// x * sigma(2u), u = sqrt(2/pi) (x + 0.044715 x^3), which is the same function
// as 0.5 x (1 + tanh u) without the cancellation of 1 + tanh u for x << 0.
template <int ACT>
__device__ __forceinline__ float activate(float x)
{
    if constexpr (ACT == ACT_RELU) {
        return x > 0.0f ? x : 0.0f;
    } else if constexpr (ACT == ACT_GELU_TANH) {
        const float u2 = 1.5957691216057308f * (x + 0.044715f * x * x * x);
        return x_sigmoid(x, u2);
    } else if constexpr (ACT == ACT_SILU) {
        return x_sigmoid(x, x);
    } else {
        return x;
    }
}

__device__ __forceinline__ float activate_dyn(float x, int act)
{
    switch (act) {
    case ACT_RELU: return activate<ACT_RELU>(x);
    case ACT_GELU_TANH: return activate<ACT_GELU_TANH>(x);
    case ACT_SILU: return activate<ACT_SILU>(x);
    default: return x;
    }
}

// Two fp32 -> packed bf16 pair, round to nearest even (hardware convert).
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi)
{
    f32x2 v = {lo, hi};
    bf16x2 h = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(unsigned int, h);
}

__device__ __forceinline__ float bf16_bits_to_float(unsigned short h)
{
    return __builtin_bit_cast(float, ((unsigned int)h) << 16);
}

// Workgroup id -> logical work item so that consecutive logical items run on
// the same XCD.  Hardware deals workgroups round-robin over the 8 XCDs, each
// with its own L2; XCD x receives ids x, x+8, ... and is given the contiguous
// logical range that starts at base(x).  Bijective for every `total`.
__device__ __forceinline__ unsigned int xcd_remap(unsigned int id, unsigned int total)
{
    const unsigned int xcd = id & 7u, q = id >> 3;
    const unsigned int per = total >> 3, rem = total & 7u;
    const unsigned int base = xcd * per + (xcd < rem ? xcd : rem);
    return base + q;
}

// Logical tile index -> (tile_m, tile_n): groups of `group_m` tile rows are
// walked column by column, so tiles that run together share A rows and B columns.
__device__ __forceinline__ void tile_coords(unsigned int r, int tiles_m, int tiles_n, int group_m,
                                            int& tm, int& tn)
{
    const unsigned int per_group = (unsigned int)group_m * (unsigned int)tiles_n;
    const unsigned int g = r / per_group;
    const unsigned int in = r - g * per_group;
    const int first = (int)g * group_m;
    const int h = (tiles_m - first) < group_m ? (tiles_m - first) : group_m;
    tn = (int)(in / (unsigned int)h);
    tm = first + (int)(in - (unsigned int)tn * (unsigned int)h);
}

}  // namespace pgk
#endif
