// Matrix-core GEMM kernels on the operand views of a convolution (a sum over the taps of GEMMs
// on shifted views of the input; see pgk_conv1d): instances and launcher.  B is always [K][N]
// here, and the tile shapes are the ones the convolution plan chooses from.
#include "pgk_gemm_mfma_kernel.h"

namespace pgk {

hipError_t launch_gemm_mfma_conv(const GemmArgs& a, int dtype, int kind, int out_mode, hipStream_t s)
{
    if (a.b_trans || a.k_rotate || out_mode != 0) return hipErrorInvalidValue;
    if (dtype == DT_BF16) {
        switch (kind) {
        case TILE_LARGE: return launch_cfg<CfgBF16, VIEW_CONV>(a, out_mode, s);
        case TILE_SMALL: return launch_cfg<CfgBF16Small, VIEW_CONV>(a, out_mode, s);
        case TILE_TALL: return launch_cfg<CfgBF16Tall, VIEW_CONV>(a, out_mode, s);
        case TILE_WIDE: return launch_cfg<CfgBF16Wide, VIEW_CONV>(a, out_mode, s);
        case TILE_FLAT: return launch_cfg<CfgBF16Flat, VIEW_CONV>(a, out_mode, s);
        default: return hipErrorInvalidValue;
        }
    }
    switch (kind) {
    case TILE_LARGE: return launch_cfg<CfgF32, VIEW_CONV>(a, out_mode, s);
    case TILE_SMALL: return launch_cfg<CfgF32Small, VIEW_CONV>(a, out_mode, s);
    case TILE_FLAT: return launch_cfg<CfgF32Flat, VIEW_CONV>(a, out_mode, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace pgk
