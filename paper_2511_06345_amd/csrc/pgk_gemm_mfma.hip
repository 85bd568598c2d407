// Matrix-core GEMM kernels, plain operand views: instances, tile table and launcher.
// The kernel template is in pgk_gemm_mfma_kernel.h.
#include "pgk_gemm_mfma_kernel.h"

namespace pgk {

bool mfma_has_tile(int dtype, int kind, bool b_trans)
{
    if (kind == TILE_LARGE || kind == TILE_SMALL || kind == TILE_FLAT) return true;
    if (kind == TILE_NARROW) return b_trans;
    if (kind == TILE_TINY) return dtype == DT_F32 && !b_trans;
    return (kind == TILE_TALL || kind == TILE_WIDE) && dtype == DT_BF16;   // (either layout of B)
}

TileShape mfma_tile_shape(int dtype, int kind)
{
    if (kind == TILE_TINY && dtype == DT_F32) return tiny_tile_shape();
    if (kind == TILE_NARROW)
        return dtype == DT_BF16 ? TileShape{CfgBF16NarrowT::BM, CfgBF16NarrowT::BN, CfgBF16NarrowT::BK}
                                : TileShape{CfgF32NarrowT::BM, CfgF32NarrowT::BN, CfgF32NarrowT::BK};
    if (kind == TILE_FLAT)
        return dtype == DT_BF16 ? TileShape{CfgBF16Flat::BM, CfgBF16Flat::BN, CfgBF16Flat::BK}
                                : TileShape{CfgF32Flat::BM, CfgF32Flat::BN, CfgF32Flat::BK};
    if (dtype == DT_BF16) {
        if (kind == TILE_TALL) return TileShape{CfgBF16Tall::BM, CfgBF16Tall::BN, CfgBF16Tall::BK};
        if (kind == TILE_WIDE) return TileShape{CfgBF16Wide::BM, CfgBF16Wide::BN, CfgBF16Wide::BK};
        return kind == TILE_SMALL ? TileShape{CfgBF16Small::BM, CfgBF16Small::BN, CfgBF16Small::BK}
                                  : TileShape{CfgBF16::BM, CfgBF16::BN, CfgBF16::BK};
    }
    return kind == TILE_SMALL ? TileShape{CfgF32Small::BM, CfgF32Small::BN, CfgF32Small::BK}
                              : TileShape{CfgF32::BM, CfgF32::BN, CfgF32::BK};
}

hipError_t launch_gemm_mfma(const GemmArgs& a, int dtype, int kind, int out_mode, hipStream_t s)
{
    if (!mfma_has_tile(dtype, kind, a.b_trans != 0)) return hipErrorInvalidValue;
    // a convolution's operand views (one bias per row marks them) have instances of their own
    if (a.bias_per_row) return launch_gemm_mfma_conv(a, dtype, kind, out_mode, s);
    if (a.b_tiles_per_tap != 0x7fffffff || a.b_col_shift != 0 || a.edge_B[0] || a.b_use_tap_table) return hipErrorInvalidValue;
    if (kind == TILE_TINY) return out_mode == 0 ? launch_gemm_tiny(a, s) : hipErrorInvalidValue;
    const bool small = kind == TILE_SMALL;
    if (kind == TILE_NARROW) return dtype == DT_BF16 ? launch_cfg<CfgBF16NarrowT, VIEW_GEMM>(a, out_mode, s) : launch_cfg<CfgF32NarrowT, VIEW_GEMM>(a, out_mode, s);
    if (kind == TILE_FLAT) {
        if (dtype == DT_BF16) return a.b_trans ? launch_cfg<CfgBF16FlatT, VIEW_GEMM>(a, out_mode, s) : launch_cfg<CfgBF16Flat, VIEW_GEMM>(a, out_mode, s);
        return a.b_trans ? launch_cfg<CfgF32FlatT, VIEW_GEMM>(a, out_mode, s) : launch_cfg<CfgF32Flat, VIEW_GEMM>(a, out_mode, s);
    }
    if (kind == TILE_TALL) return a.b_trans ? launch_cfg<CfgBF16TallT, VIEW_GEMM>(a, out_mode, s) : launch_cfg<CfgBF16Tall, VIEW_GEMM>(a, out_mode, s);
    if (kind == TILE_WIDE) return a.b_trans ? launch_cfg<CfgBF16WideT, VIEW_GEMM>(a, out_mode, s) : launch_cfg<CfgBF16Wide, VIEW_GEMM>(a, out_mode, s);
    if (a.b_trans) {
        if (dtype == DT_BF16) return small ? launch_cfg<CfgBF16SmallT, VIEW_GEMM>(a, out_mode, s) : launch_cfg<CfgBF16T, VIEW_GEMM>(a, out_mode, s);
        return small ? launch_cfg<CfgF32SmallT, VIEW_GEMM>(a, out_mode, s) : launch_cfg<CfgF32T, VIEW_GEMM>(a, out_mode, s);
    }
    if (dtype == DT_BF16) return small ? launch_cfg<CfgBF16Small, VIEW_GEMM>(a, out_mode, s) : launch_cfg<CfgBF16, VIEW_GEMM>(a, out_mode, s);
    return small ? launch_cfg<CfgF32Small, VIEW_GEMM>(a, out_mode, s) : launch_cfg<CfgF32, VIEW_GEMM>(a, out_mode, s);
}

hipError_t launch_gemm_mfma_timed(const GemmArgs& a, int dtype, hipStream_t s)
{
    if (a.b_trans || a.bias_per_row || a.splits != 1 || !a.stamps) return hipErrorInvalidValue;
    return dtype == DT_BF16 ? launch_cfg<CfgBF16, VIEW_GEMM, true>(a, 0, s) : launch_cfg<CfgF32, VIEW_GEMM, true>(a, 0, s);
}

}  // namespace pgk
