// Matrix-core GEMM main loop with the fused epilogue, for gfx950 (MI355X): the kernel template
// and its shipping configurations.  Included by the two files that instantiate it
// (pgk_gemm_mfma.hip: plain GEMM operands; pgk_gemm_mfma_conv.hip: convolution views).
//
// The operator is the textbook one the paper's matmul / activation / reduction
// categories refer to (PRAGMA Sections 1 and 4.2): C = act(A*B + bias) with an
// optional row sum.  Everything about how it is computed below is this
// library's own design for CDNA4:
//
//  * One workgroup owns a BM x BN tile of C.  A and B tiles of BK along K are
//    copied global -> LDS with 128-bit direct-to-LDS loads into rings of two
//    (or, for the A tiles of the bf16 kernels, three) stages, so the copies of the
//    next tiles overlap the matrix-core work on tile kt.
//  * LDS rows are stored in 16-byte chunks whose position is XOR-swizzled with
//    the row index; the direct-to-LDS write is always one contiguous 1 KiB per
//    wave instruction, so the swizzle is applied by choosing which global chunk
//    each lane fetches.
//  * MFMA operand roles are swapped (the B-matrix columns feed the "A" operand
//    and the A-matrix rows the "B" operand), so the accumulator tile a lane holds
//    is one row of C with runs of 4 consecutive columns.  Row sums are then
//    mostly in-lane adds, bias loads and C stores are 4 elements wide.
//  * bf16: v_mfma_f32_16x16x32_bf16.  A rows are K-contiguous in LDS
//    (ds_read_b128); B is N-contiguous, so its operand is gathered with the
//    transposing ds_read_b64_tr_b16.  Of the two bf16 shapes this one reads and
//    writes half as many accumulator registers per multiply-add (a 16 x 16 block
//    per 32 k values instead of a 32 x 32 block per 16), and under the board's power
//    limit that shows as clock: matrix instructions alone on random register
//    operands sustain 2230 TFLOP/s with it against 1940 with 32 x 32 x 16, the
//    8192^3 GEMM 764 against 837 us on the same machine.
//  * fp32: v_mfma_f32_32x32x2_f32 (at a sixteenth of the bf16 rate the matrix
//    pipes are not what the power limit sees).
//  * Workgroup ids are remapped so that each XCD (own L2) works on a compact
//    group of tiles.
#ifndef PGK_GEMM_MFMA_KERNEL_H
#define PGK_GEMM_MFMA_KERNEL_H

#include <hip/hip_runtime.h>

#include <cstddef>
#include <type_traits>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

template <bool BT_, bool BF16_, int BM_, int BN_, int BK_, int WGM_, int WGN_, int A_STAGES_, int WAVES_PER_SIMD_>
struct MfmaCfgBase {
    static constexpr bool BF16 = BF16_;
    // B given transposed, [N][K] with K contiguous (a linear layer's weight as stored): its
    // tile then sits in LDS like the A tile, [BN][BK], and is fetched like it
    static constexpr bool BT = BT_;
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
    // LDS ring depth of the A tiles (2 or 3); the B tiles always have 2 stages.  With 3,
    // the copy of an A tile is issued a whole K tile earlier than it is needed, so only
    // the B half of the traffic has to land within one tile's worth of MFMAs.
    static constexpr int A_STAGES = A_STAGES_;
    // waves the register allocation must leave room for on one SIMD
    static constexpr int WAVES_PER_SIMD = WAVES_PER_SIMD_;
    static constexpr int ES = BF16_ ? 2 : 4;       // element bytes
    static constexpr int NW = WGM * WGN;           // waves per workgroup
    static constexpr int NT = NW * 64;             // threads per workgroup
    static constexpr int WM = BM / WGM;            // rows per wave
    static constexpr int WN = BN / WGN;            // cols per wave
    static constexpr int TM = WM / 32, TN = WN / 32;   // 32 x 32 accumulator blocks per wave (fp32 instruction)
    // bf16 uses the 16 x 16 x 32 instruction: 16 x 16 blocks; the B fragments of a step of 32 along
    // K are fetched and used in groups of JG blocks -- half of the wave's columns, at least two
    // blocks -- which bounds the registers the operand double buffers take and gives a K tile
    // four sub-steps (two on the skinny tiles), so that the wait for the next tile's copies
    // (before the last one) comes three quarters of the way through the tile
    static constexpr int TM16 = WM / 16, TN16 = WN / 16;
    static constexpr int JG = TN16 > 2 ? TN16 / 2 : TN16, NJH = TN16 / JG;
    static constexpr int RA = BK * ES;             // LDS row bytes of the A tile
    static constexpr int RB = BT ? BK * ES : BN * ES;   // LDS row bytes of the B tile
    static constexpr int A_BYTES = BM * RA, B_BYTES = BN * BK * ES;
    static constexpr int A_CPW = A_BYTES / 1024 / NW;  // 1 KiB copy instructions per wave
    static constexpr int B_CPW = B_BYTES / 1024 / NW;
    static constexpr int A_CPR = RA / 16, B_CPR = RB / 16;  // 16 B chunks per row
    static constexpr int A_RPC = 1024 / RA, B_RPC = 1024 / RB;  // rows per 1 KiB
    static constexpr int LDS_BYTES = A_STAGES * A_BYTES + 2 * B_BYTES;
    // the epilogue stages the output tile in the operand buffers, in pieces the size of the
    // larger kind (the B stages first when the B tile is the larger one: skinny-M tiles)
    static constexpr bool STAGE_IN_B = B_BYTES > A_BYTES;
    static constexpr int PIECE_BYTES = STAGE_IN_B ? B_BYTES : A_BYTES;
    static_assert(A_STAGES == 2 || A_STAGES == 3, "A ring depth");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of one CU");
    static_assert(RA == 128 || RA == 64, "A-tile swizzle assumes 128- or 64-byte rows");
    static_assert(BT || RB % 256 == 0, "B-tile swizzle assumes rows of a multiple of 256 bytes");
    static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile / wave split");
    static_assert(BM <= NT, "row-sum combine uses one thread per tile row");
};
// <bf16, BM, BN, BK, wave rows, wave cols, A ring depth, waves/SIMD>: B as [K][N] ...
template <bool BF16_, int BM_, int BN_, int BK_, int WGM_, int WGN_, int A_STAGES_, int WAVES_PER_SIMD_>
struct MfmaCfg : MfmaCfgBase<false, BF16_, BM_, BN_, BK_, WGM_, WGN_, A_STAGES_, WAVES_PER_SIMD_> {};
// ... and B given transposed, [N][K]
template <bool BF16_, int BM_, int BN_, int BK_, int WGM_, int WGN_, int A_STAGES_, int WAVES_PER_SIMD_>
struct MfmaCfgBt : MfmaCfgBase<true, BF16_, BM_, BN_, BK_, WGM_, WGN_, A_STAGES_, WAVES_PER_SIMD_> {};

// A tile: rows of CPR chunks; 16 consecutive rows read the same logical chunk
// at once, so the 16 chunk slots of a 256-byte bank period must all differ.
template <int CPR>
__device__ __forceinline__ int swz_a(int row) { return (row / (16 / CPR)) % CPR; }
template <bool BF16>
__device__ __forceinline__ int swz_b(int krow)
{
    // bf16: the transposing read of a 16-lane group touches 4 consecutive k rows, and the two
    // groups that are served together sit 8 rows apart; fp32: the two half-waves read rows 4 apart.
    return BF16 ? (4 * (krow & 3)) ^ (2 * ((krow >> 3) & 1)) : 8 * ((krow >> 2) & 1);
}

// Epilogues.  A lane's accumulators are rows of C in runs of 4 consecutive columns; such a run is
// one "unit" (16 bytes as fp32, 8 as bf16).  Bias, activation, rounding and the row-sum
// contribution are applied to the accumulators, the output goes through LDS (the operand buffers
// of the main loop, free by then) to turn units into whole row pieces, and is stored as 16-byte
// chunks.  Two forms: per wave (epilogue_wave32, epilogue_wave16 below: every wave on its own
// part of the tile, no workgroup barrier) wherever a wave's row pieces are whole 128-byte lines,
// and workgroup-wide (epilogue_to_lds16 + epilogue_store: stage the whole tile, barrier, store
// whole tile rows) for the bf16 tiles whose waves own 32 columns.
// `bias` / `bias_row`: this tile's column or row biases, already in LDS (see the kernel).
// KIND: EPI_PLAIN -- column bias only, no row sum: the per-element work is one add, the
// activation and the rounding (the large GEMMs' case); EPI_ROWSUM -- plus the row sums of a
// full tile; EPI_ROWSUM_MASKED -- the same for a last tile column that is not full (columns
// past the end of N add nothing); EPI_ROWBIAS -- column biases are zero, one bias per row
// (bias_row), no row sum.
// HAS_BIAS false: `bias` is not read (the split-K partial products).
enum { EPI_PLAIN = 0, EPI_ROWSUM = 1, EPI_ROWSUM_MASKED = 2, EPI_ROWBIAS = 3 };

// Workgroup-wide staging of a bf16 tile whose accumulators are 16 x 16 blocks (v_mfma_f32_16x16x32_bf16
// with the operand roles swapped): lane (l16 = lane % 16, grp = lane / 16) holds, of block (i, j)
// of its wave's part, row 16 i + l16 and the four columns 16 j + 4 grp ..: one unit per block.
// Output is bf16.  The tile is spread over (up to) four operand buffers, whole rows of BN
// elements each; inside a row the unit index is XORed with twice the row index, so that the
// sixteen rows and four units a wave writes at once fall in different banks, and so that the
// pair of units forming a 16-byte chunk stays adjacent for epilogue_store.
template <int ACT, int KIND, typename Cfg, bool HAS_BIAS = true>
__device__ __forceinline__ void epilogue_to_lds16(f32x4 (&acc)[Cfg::TM16][Cfg::TN16], const float* bias,
                                                  const float* bias_row,
                                                  int n_rem, int wm, int wn, int lane,
                                                  unsigned char* const (&obj)[4], float* rs_lds)
{
    constexpr int TM16 = Cfg::TM16, TN16 = Cfg::TN16;
    constexpr int UB = 8;                                 // bytes per unit
    constexpr int ROW_BYTES = Cfg::BN * 2;
    constexpr int UNITS = ROW_BYTES / UB;                 // units per row
    constexpr int ROWS_PER_OBJ = Cfg::PIECE_BYTES / ROW_BYTES;   // output rows one operand buffer holds
    constexpr bool ROWSUM = KIND == EPI_ROWSUM || KIND == EPI_ROWSUM_MASKED;
    const int grp = lane >> 4;
    const int row_in = lane & 15;
#pragma unroll
    for (int i = 0; i < TM16; ++i) {
        float rs = 0.0f;
        const int row = wm * Cfg::WM + 16 * i + row_in;   // row inside the tile
        const int o = (wm * Cfg::WM + 16 * i) / ROWS_PER_OBJ;
        unsigned char* base = (o == 0 ? obj[0] : o == 1 ? obj[1] : o == 2 ? obj[2] : obj[3]) +
                              (row % ROWS_PER_OBJ) * ROW_BYTES;
        const int key = (2 * row) % UNITS;
        float br = 0.0f;
        if constexpr (KIND == EPI_ROWBIAS) br = bias_row[row];
#pragma unroll
        for (int j = 0; j < TN16; ++j) {
            const int col = wn * Cfg::WN + 16 * j + 4 * grp;   // column inside the tile
            f32x4 bv;
            if constexpr (HAS_BIAS && KIND != EPI_ROWBIAS) bv = *(const f32x4*)(bias + col);
            else bv = f32x4{br, br, br, br};
            float y[4];
            // columns past the end of a ragged N add nothing to the row sum: `left` of this
            // unit's four exist.  (Kept opaque, so that each comparison is made where it is
            // used: hoisted out of the loops, the lane masks of a wave's outputs would live in
            // scalar registers and spill.)
            int left = n_rem - col;
            if constexpr (KIND == EPI_ROWSUM_MASKED) asm volatile("" : "+v"(left));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                y[e] = activate<ACT>(acc[i][j][e] + bv[e]);
                if constexpr (KIND == EPI_ROWSUM) rs += y[e];
                else if constexpr (KIND == EPI_ROWSUM_MASKED) rs += e < left ? y[e] : 0.0f;
            }
            unsigned char* dst = base + (((col >> 2) ^ key) * UB);
            u32x2 pk = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
            *(u32x2*)dst = pk;
            // keeps the bias fetches of later blocks below this block's work
            if (j % 4 == 3) asm volatile("" ::: "memory");
        }
        if constexpr (ROWSUM) {
            // the four lanes that share a row, in a fixed order
            rs += __shfl_xor(rs, 16);
            rs += __shfl_xor(rs, 32);
            if (grp == 0) rs_lds[wn * Cfg::BM + row] = rs;
        }
    }
}

// The bf16 epilogue of the tiles whose waves own at least 64 columns (row pieces of 128 bytes
// and more): every wave stages and stores its own part of the tile, sixteen rows at a time, with
// no workgroup barrier -- bias + activation + rounding of a 16-row block into a piece of LDS that
// only this wave touches (the LDS operations of one wave are carried out in order), read back as
// 16-byte chunks of whole row pieces, stored, and on to the next block while those stores drain.
// A wave instruction stores 64 x 16 bytes = complete 128-byte lines of 4 (or 8) consecutive rows.
// The activation arithmetic of a block so overlaps the stores of the one before, where the
// workgroup-wide form (stage everything, barrier, store everything) adds the two up.
// Staging layout of a block: [16 rows][WN columns] bf16, the 8-byte unit index XORed with a key of
// the row (rows that share a 256-byte bank period share the key), so that the sixteen rows and
// four units a wave writes at once, and the row pieces it reads back, fall in different banks.
// Row sums as in the workgroup-wide form: per-wave partials to rs_lds, combined by the caller
// after a barrier.
template <int ACT, int KIND, typename Cfg, bool HAS_BIAS = true>
__device__ __forceinline__ void epilogue_wave16(f32x4 (&acc)[Cfg::TM16][Cfg::TN16], const float* bias,
                                                const float* bias_row, unsigned char* out_tile, size_t ld_bytes,
                                                int m_rem, int n_rem, int wm, int wn, int wave, int lane,
                                                unsigned char* const (&obj)[4], float* rs_lds)
{
    constexpr int TM16 = Cfg::TM16, TN16 = Cfg::TN16;
    constexpr int ROWB = Cfg::WN * 2;                     // bytes of a row piece
    constexpr int UNITS = ROWB / 8;                       // 8-byte units per row piece
    constexpr int RPP = ROWB >= 256 ? 1 : 256 / ROWB;     // rows per 256-byte bank period
    constexpr int BLK = 16 * ROWB;                        // bytes of a staged block
    constexpr int WAVE_BYTES = TM16 * BLK;                // all blocks of a wave
    constexpr int WPP = Cfg::PIECE_BYTES / WAVE_BYTES;    // waves per operand buffer
    constexpr int CPR = ROWB / 16;                        // 16-byte chunks per row piece
    constexpr int CH = 16 * CPR / 64;                     // chunks per lane and block
    static_assert(ROWB >= 128 && Cfg::PIECE_BYTES % WAVE_BYTES == 0 && Cfg::NW <= 4 * WPP && 16 * CPR % 64 == 0,
                  "row pieces of whole lines; the operand buffers hold every wave's blocks");
    constexpr bool ROWSUM = KIND == EPI_ROWSUM || KIND == EPI_ROWSUM_MASKED;
    const int grp = lane >> 4;
    const int row_in = lane & 15;
    const int o = wave / WPP;
    unsigned char* const mine = (o == 0 ? obj[0] : o == 1 ? obj[1] : o == 2 ? obj[2] : obj[3]) + (wave % WPP) * WAVE_BYTES;
    const int wkey = (2 * (row_in / RPP)) % UNITS;        // key of the row this lane writes
    using chunk_at_element = u32x4_align2;
#pragma unroll
    for (int i = 0; i < TM16; ++i) {
        unsigned char* const blk = mine + i * BLK;
        const int row = wm * Cfg::WM + 16 * i + row_in;   // row inside the tile
        float rs = 0.0f;
        float br = 0.0f;
        if constexpr (KIND == EPI_ROWBIAS) br = bias_row[row];
#pragma unroll
        for (int j = 0; j < TN16; ++j) {
            const int colw = 16 * j + 4 * grp;            // column inside the wave's part
            const int col = wn * Cfg::WN + colw;          // ... inside the tile
            f32x4 bv;
            if constexpr (HAS_BIAS && KIND != EPI_ROWBIAS) bv = *(const f32x4*)(bias + col);
            else bv = f32x4{br, br, br, br};
            float y[4];
            int left = n_rem - col;
            if constexpr (KIND == EPI_ROWSUM_MASKED) asm volatile("" : "+v"(left));
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                y[e] = activate<ACT>(acc[i][j][e] + bv[e]);
                if constexpr (KIND == EPI_ROWSUM) rs += y[e];
                else if constexpr (KIND == EPI_ROWSUM_MASKED) rs += e < left ? y[e] : 0.0f;
            }
            u32x2 pk = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
            *(u32x2*)(blk + row_in * ROWB + (((colw >> 2) ^ wkey) * 8)) = pk;
            if (j % 4 == 3) asm volatile("" ::: "memory");
        }
        if constexpr (ROWSUM) {
            rs += __shfl_xor(rs, 16);
            rs += __shfl_xor(rs, 32);
            if (grp == 0) rs_lds[wn * Cfg::BM + row] = rs;
        }
        // the block's row pieces, 16 bytes per lane and instruction, back from LDS and out
        u32x4 v[CH];
#pragma unroll
        for (int t = 0; t < CH; ++t) {
            const int c = lane + 64 * t;
            const int r = c / CPR, cc = c % CPR;
            const int key = (2 * (r / RPP)) % UNITS;
            v[t] = *(const u32x4*)(blk + r * ROWB + (((2 * cc) ^ key) * 8));
        }
#pragma unroll
        for (int t = 0; t < CH; ++t) {
            const int c = lane + 64 * t;
            const int r = c / CPR, cc = c % CPR;
            const int trow = wm * Cfg::WM + 16 * i + r;
            const int left = n_rem - (wn * Cfg::WN + cc * 8);     // elements of this chunk that exist
            if (trow >= m_rem || left <= 0) continue;
            unsigned char* at = out_tile + (size_t)trow * ld_bytes + (size_t)(wn * Cfg::WN) * 2 + (size_t)cc * 16;
            if (left >= 8) {
                __builtin_nontemporal_store(v[t], (chunk_at_element*)at);
            } else {
#pragma unroll
                for (int e = 0; e < 7; ++e) {
                    if (e >= left) break;
                    const unsigned int word = v[t][e / 2];
                    ((unsigned short*)at)[e] = (unsigned short)(e % 2 ? word >> 16 : word & 0xffffu);
                }
            }
        }
    }
}

// The per-wave epilogue of the fp32 kernels (32 x 32 accumulator blocks: lane (l32, half) holds,
// of block (i, j), row 32 i + l32 and the columns 32 j + 8 g + 4 half .., g = 0..3; a unit is 16
// bytes): a wave's row pieces are 128 or 256 bytes for every fp32 tile shape, so all of them
// take this form.  STREAM: non-temporal stores (C); plain ones for split-K partial products,
// which the second pass reads back soon.
template <int ACT, int KIND, typename Cfg, bool HAS_BIAS, bool STREAM>
__device__ __forceinline__ void epilogue_wave32(f32x16 (&acc)[Cfg::TM][Cfg::TN], const float* bias,
                                                const float* bias_row, unsigned char* out_tile, size_t ld_bytes,
                                                int m_rem, int n_rem, int wm, int wn, int wave, int lane,
                                                unsigned char* const (&obj)[4], float* rs_lds)
{
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    constexpr int ROWB = Cfg::WN * 4;                     // bytes of a row piece
    constexpr int UNITS = ROWB / 16;                      // 16-byte units (= chunks) per row piece
    constexpr int RPP = ROWB >= 256 ? 1 : 256 / ROWB;     // rows per 256-byte bank period
    constexpr int BLK = 32 * ROWB;                        // bytes of a staged block
    constexpr int WAVE_BYTES = TM * BLK;
    constexpr int WPP = Cfg::PIECE_BYTES / WAVE_BYTES;    // waves per operand buffer
    constexpr int CH = 32 * UNITS / 64;                   // chunks per lane and block
    static_assert(ROWB >= 128 && Cfg::PIECE_BYTES % WAVE_BYTES == 0 && Cfg::NW <= 4 * WPP && (32 * UNITS) % 64 == 0,
                  "row pieces of whole lines; the operand buffers hold every wave's blocks");
    constexpr bool ROWSUM = KIND == EPI_ROWSUM || KIND == EPI_ROWSUM_MASKED;
    const int half = lane >> 5;
    const int row_in = lane & 31;
    const int o = wave / WPP;
    unsigned char* const mine = (o == 0 ? obj[0] : o == 1 ? obj[1] : o == 2 ? obj[2] : obj[3]) + (wave % WPP) * WAVE_BYTES;
    const int wkey = (row_in / RPP) % UNITS;              // key of the row this lane writes
    using chunk_at_element = u32x4_align4;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        unsigned char* const blk = mine + i * BLK;
        const int row = wm * Cfg::WM + 32 * i + row_in;   // row inside the tile
        float rs = 0.0f;
        float br = 0.0f;
        if constexpr (KIND == EPI_ROWBIAS) br = bias_row[row];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            f32x4 bvs[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if constexpr (HAS_BIAS && KIND != EPI_ROWBIAS) bvs[g] = *(const f32x4*)(bias + wn * Cfg::WN + 32 * j + 8 * g + 4 * half);
                else bvs[g] = f32x4{br, br, br, br};
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int colw = 32 * j + 8 * g + 4 * half;   // column inside the wave's part
                int left = n_rem - (wn * Cfg::WN + colw);
                if constexpr (KIND == EPI_ROWSUM_MASKED) asm volatile("" : "+v"(left));
                f32x4 y;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    y[e] = activate<ACT>(acc[i][j][4 * g + e] + bvs[g][e]);
                    if constexpr (KIND == EPI_ROWSUM) rs += y[e];
                    else if constexpr (KIND == EPI_ROWSUM_MASKED) rs += e < left ? y[e] : 0.0f;
                }
                *(f32x4*)(blk + row_in * ROWB + (((colw >> 2) ^ wkey) * 16)) = y;
            }
            asm volatile("" ::: "memory");
        }
        if constexpr (ROWSUM) {
            rs += __shfl_xor(rs, 32);
            if (half == 0) rs_lds[wn * Cfg::BM + row] = rs;
        }
        u32x4 v[CH];
#pragma unroll
        for (int t = 0; t < CH; ++t) {
            const int c = lane + 64 * t;
            const int r = c / UNITS, cc = c % UNITS;
            v[t] = *(const u32x4*)(blk + r * ROWB + ((cc ^ ((r / RPP) % UNITS)) * 16));
        }
#pragma unroll
        for (int t = 0; t < CH; ++t) {
            const int c = lane + 64 * t;
            const int r = c / UNITS, cc = c % UNITS;
            const int trow = wm * Cfg::WM + 32 * i + r;
            const int left = n_rem - (wn * Cfg::WN + cc * 4);     // elements of this chunk that exist
            if (trow >= m_rem || left <= 0) continue;
            unsigned char* at = out_tile + (size_t)trow * ld_bytes + (size_t)(wn * Cfg::WN) * 4 + (size_t)cc * 16;
            if (left >= 4) {
                if constexpr (STREAM) __builtin_nontemporal_store(v[t], (chunk_at_element*)at);
                else *(chunk_at_element*)at = v[t];
            } else {
#pragma unroll
                for (int e = 0; e < 3; ++e) {
                    if (e >= left) break;
                    ((unsigned int*)at)[e] = v[t][e];
                }
            }
        }
    }
}

// Epilogue, part 2: the staged tile goes to global memory as whole rows: a wave
// instruction stores 64 x 16 bytes = complete 128-byte lines of consecutive rows.
// STREAM: the output is not read again soon (C, as opposed to split-K partial products):
// non-temporal stores, which leave the operand panels in L2 alone (measured with rotating
// buffers: 8192 x 8192 x 1024 bf16 176 -> 166 us, x 8192 809 -> 803 us, conv1d 524 -> 509 us).
template <bool OUT_BF16, typename Cfg, bool STREAM>
__device__ __forceinline__ void epilogue_store(unsigned char* out_tile, size_t ld_bytes, int tid,
                                               int m_rem, int n_rem, unsigned char* const (&obj)[4])
{
    constexpr int ROW_BYTES = Cfg::BN * (OUT_BF16 ? 2 : 4);
    constexpr int CPR = ROW_BYTES / 16;                   // 16-byte chunks per row
    constexpr int UB = OUT_BF16 ? 8 : 16;
    constexpr int UNITS = ROW_BYTES / UB;
    constexpr int ROWS_PER_OBJ = Cfg::PIECE_BYTES / ROW_BYTES;   // output rows one operand buffer holds
    constexpr int ROWS_PER_IT = Cfg::NT / CPR;
    constexpr int ITERS = Cfg::BM / ROWS_PER_IT;
    static_assert(ROWS_PER_OBJ % ROWS_PER_IT == 0, "an iteration stays inside one buffer");
    const int c = tid % CPR;
    // all of the thread's chunks are read from LDS first (one round trip), then stored; the
    // scheduling barrier keeps the compiler from sinking each read into its store's branch
    u32x4 v[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int row = it * ROWS_PER_IT + tid / CPR;
        const int o = (it * ROWS_PER_IT) / ROWS_PER_OBJ;  // compile-time after unrolling
        const unsigned char* base = (o == 0 ? obj[0] : o == 1 ? obj[1] : o == 2 ? obj[2] : obj[3]) +
                                    (row % ROWS_PER_OBJ) * ROW_BYTES;
        const int key = (2 * row) % UNITS;
        const int unit = OUT_BF16 ? ((2 * c) ^ key) : (c ^ key);
        v[it] = *(const u32x4*)(base + unit * UB);
    }
    __builtin_amdgcn_sched_barrier(0);
    // N need not be a multiple of the 16-byte chunk: the row's last chunk may hold fewer
    // elements, which are then stored one by one, and rows start on element boundaries only
    // (the 16-byte stores are declared with that alignment; global memory takes them as they are)
    using chunk_at_element = typename std::conditional<OUT_BF16, u32x4_align2, u32x4_align4>::type;
    constexpr int EPC = 16 / (OUT_BF16 ? 2 : 4);
    const int left = n_rem - c * EPC;                  // elements of this chunk that exist
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int row = it * ROWS_PER_IT + tid / CPR;
        if (row >= m_rem || left <= 0) continue;
        unsigned char* at = out_tile + (size_t)row * ld_bytes + (size_t)c * 16;
        if (left >= EPC) {
            if constexpr (STREAM) __builtin_nontemporal_store(v[it], (chunk_at_element*)at);
            else *(chunk_at_element*)at = v[it];
        } else {
#pragma unroll
            for (int e = 0; e < EPC - 1; ++e) {
                if (e >= left) break;
                const unsigned int word = v[it][OUT_BF16 ? e / 2 : e];
                if constexpr (OUT_BF16) ((unsigned short*)at)[e] = (unsigned short)(e % 2 ? word >> 16 : word & 0xffffu);
                else ((unsigned int*)at)[e] = word;
            }
        }
    }
}

template <int V>
struct IC { static constexpr int value = V; };

// VIEW: how the operands are addressed.  VIEW_GEMM: plain dense operands (optionally a transposed
// B, a K rotation, ragged rows).  VIEW_CONV: a convolution read as a sum of shifted GEMMs --
// A shared by the batch entries, B tiles that walk tap after tap over the input channels, edge
// tile columns that read zero-padded strips, one bias per row.  The plain instances carry none of
// the convolution's address state.
enum { VIEW_GEMM = 0, VIEW_CONV = 1 };

// TIMED: a measurement instance (see pgk_probe_gemm_phases): wave 0 of every workgroup writes
// the shader-clock cycle counter and the constant 100 MHz counter at six points of the kernel to
// p.stamps[workgroup][kStampWords], and waits for its stores to be acknowledged before the last
// stamp.  The shipping instances (TIMED false) contain none of it.
template <typename Cfg, int VIEW, bool TIMED = false>
__global__ __launch_bounds__(Cfg::NT, Cfg::WAVES_PER_SIMD) void gemm_mfma_kernel(const GemmArgs p, const int out_mode)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub (and has no buffer-resource type)
    constexpr bool BF16 = Cfg::BF16;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, ES = Cfg::ES;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, RA = Cfg::RA, RB = Cfg::RB;
    // operand-fetch steps per K tile: fp32 steps of 8 along K; bf16 steps of 32, each cut into
    // NJH sub-steps over groups of JG B fragments
    constexpr int JG = Cfg::JG, NJH = Cfg::NJH;
    constexpr int NS = BF16 ? (BK / 32) * NJH : BK / 8;
    static_assert(NS % 2 == 0, "fragment double buffer assumes an even step count");

    // Separate LDS objects per stage and operand (not one array indexed by stage): the
    // compiler can then tell that a direct-to-LDS copy into one stage does not alias
    // the operand reads of another stage, and does not make those reads wait for it.
    constexpr int SA = Cfg::A_STAGES;
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a0[Cfg::A_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a1[Cfg::A_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a2[SA > 2 ? Cfg::A_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_b0[Cfg::B_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_b1[Cfg::B_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / Cfg::WGN, wn = wave % Cfg::WGN;
    // phase stamp k of this workgroup: (cycles, 100 MHz ticks)
    auto stamp = [&](int k) __attribute__((always_inline)) {
        if constexpr (TIMED) {
            __builtin_amdgcn_sched_barrier(0);
            const unsigned long long cyc = __builtin_readcyclecounter();
            const unsigned long long tick = __builtin_amdgcn_s_memrealtime();
            // (all lanes of wave 0 store the same two words: a wave-uniform branch, so that the
            // code after it is not seen as reached under a divergent condition)
            if (wave == 0) {
                unsigned long long* at = p.stamps + (size_t)blockIdx.x * kStampWords + 2 * k;
                at[0] = cyc;
                at[1] = tick;
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    stamp(0);
    if constexpr (TIMED) {
        // where the workgroup runs: hardware id register (CU, shader engine) and XCD number
        if (wave == 0) {
            p.stamps[(size_t)blockIdx.x * kStampWords + 12] = (unsigned long long)__builtin_amdgcn_s_getreg(63492);   // HW_ID, 32 bits
            p.stamps[(size_t)blockIdx.x * kStampWords + 13] = (unsigned long long)__builtin_amdgcn_s_getreg(63508);   // XCC_ID, 32 bits
        }
    }

    // ---- which tile, batch entry and K slice this workgroup owns
    const unsigned int tiles = (unsigned int)p.tiles_m * (unsigned int)p.tiles_n;
    const unsigned int logical = xcd_remap(blockIdx.x, gridDim.x);
    const unsigned int z = logical / tiles;
    int tm, tn;
    tile_coords(logical - z * tiles, p.tiles_m, p.tiles_n, p.group_m, tm, tn);
    const int b = (int)(z / (unsigned int)p.splits);
    const int sp = (int)(z - (unsigned int)b * (unsigned int)p.splits);
    const int k_begin = sp * p.k_slice;
    const int k_end = (k_begin + p.k_slice < p.K) ? (k_begin + p.k_slice) : p.K;
    // K tiles of this slice; the last one may be partial (K need not be a multiple of BK, nor
    // of the 16-byte chunk: operand rows only have to start on 4-byte boundaries): k_last of
    // its BK columns exist
    const int KT = (k_end - k_begin + BK - 1) / BK;
    const int k_last = (k_end - k_begin) - (KT - 1) * BK;
    // (a last tile that is full is treated the same way when the rows of a plain B are not
    // whole chunks: the copy of its last row must end where the array ends)
    const bool k_partial = k_last < BK || p.b_tail_bounded;
    // Memory-bound skinny products: every workgroup walks its K tiles from a different starting
    // tile (and wraps around).  With row strides that are large powers of two, workgroups that
    // all start at tile 0 and move in step keep asking the same few memory channels
    // (bf16 16384 x 16 x 16384, rows 32 KiB apart: 4.0 TB/s; with rows of 32896 bytes 5.4 TB/s).
    // Only with whole K tiles (the peeled partial tile has to come last) and plain GEMM views.
    // (The workgroups of one batch entry share its small operand through L2 and stay in step;
    // the batch entries start apart.  A single entry: every tile on its own.)
    const int k_rot = (VIEW == VIEW_GEMM && p.k_rotate && !k_partial) ? (int)((unsigned int)(p.batch > 1 ? b : tm + tn) % (unsigned int)KT) : 0;

    const unsigned char* Ag = (const unsigned char*)p.A +
        ((size_t)b * (size_t)p.a_batch_stride + (size_t)tm * BM * p.K + (size_t)k_begin) * ES;
    // where this tile column's B operand lives: the B array itself, its columns shifted by
    // b_col_shift (0 for a GEMM), or, for an edge tile column of a convolution, a strip
    const unsigned char* b_src = (const unsigned char*)p.B;
    int ldb = p.ldb;
    long long b_batch_stride = p.b_batch_stride;
    long long b_col0 = (long long)tn * BN;
    if constexpr (VIEW == VIEW_CONV) {
        b_col0 += p.b_col_shift;
#pragma unroll
        for (int e = 0; e < 3; ++e) {
            if (p.edge_B[e] && p.edge_tn[e] == tn) {
                b_src = (const unsigned char*)p.edge_B[e];
                ldb = p.edge_ldb;
                b_batch_stride = p.edge_batch_stride;
                b_col0 = 0;
            }
        }
    }
    // (transposed B: rows are tile columns, K runs along them)
    const unsigned char* Bg = b_src +
        (Cfg::BT ? ((long long)b * b_batch_stride + b_col0 * ldb + (long long)k_begin) * ES
                 : ((long long)b * b_batch_stride + (long long)k_begin * ldb + b_col0) * ES);
    const size_t a_step = (size_t)BK * ES;             // bytes per K tile along an A row
    const size_t b_step = Cfg::BT ? (size_t)BK * ES : (size_t)BK * ldb * ES;   // bytes per K tile of B
    // one past the last byte of A and of B: copies of a partial K tile run past the end of a
    // row (into the next row, harmless) and, for the last row, past the end of the array,
    // where the buffer resource's size check makes them read nothing
    const unsigned char* const A_end = (const unsigned char*)p.A +
        ((size_t)(p.batch - 1) * (size_t)p.a_batch_stride + (size_t)p.M * p.K) * ES;
    const unsigned char* const B_end = (const unsigned char*)p.B +
        ((size_t)(p.batch - 1) * (size_t)p.b_batch_stride + (size_t)(Cfg::BT ? p.N : p.K) * p.ldb) * ES;

    // rows / columns of this tile that exist (smaller than the tile on a ragged edge)
    const int m_rem = (p.M - tm * BM) < BM ? (p.M - tm * BM) : BM;
    const int n_rem = (p.N - tn * BN) < BN ? (p.N - tn * BN) : BN;

    // this tile's biases (one per column, or one per row), one value per thread, fetched now
    // and handed out through LDS in the epilogue
    constexpr int BIAS_N = BM > BN ? BM : BN;
    static_assert(BIAS_N <= Cfg::NT, "one thread per bias value");
    float bias_pre = 0.0f;
    constexpr bool BIAS_PER_ROW = VIEW == VIEW_CONV;
    if (p.bias && out_mode == 0) {
        if constexpr (BIAS_PER_ROW) { if (tid < m_rem) bias_pre = p.bias[(size_t)tm * BM + tid]; }
        else if (tid < n_rem) bias_pre = p.bias[(size_t)tn * BN + tid];
    }

    // ---- per-lane byte offsets of the global chunks this lane copies
    unsigned int voff_a[Cfg::A_CPW], voff_b[Cfg::B_CPW];
#pragma unroll
    for (int t = 0; t < Cfg::A_CPW; ++t) {
        const int ch = wave * Cfg::A_CPW + t;
        const int r = ch * Cfg::A_RPC + lane / Cfg::A_CPR;
        const int c = (lane % Cfg::A_CPR) ^ swz_a<Cfg::A_CPR>(r);
        // rows past the end of A (last tile row of a ragged M) re-read the last valid row:
        // they only feed output rows that are never stored
        const int rg = r < m_rem ? r : m_rem - 1;
        voff_a[t] = (unsigned int)rg * (unsigned int)p.K * ES + (unsigned int)c * 16u;
    }
#pragma unroll
    for (int t = 0; t < Cfg::B_CPW; ++t) {
        const int ch = wave * Cfg::B_CPW + t;
        if constexpr (Cfg::BT) {
            // rows of the transposed B are tile columns: same scheme as for A
            const int r = ch * Cfg::B_RPC + lane / Cfg::B_CPR;
            const int c = (lane % Cfg::B_CPR) ^ swz_a<Cfg::B_CPR>(r);
            const int rg = r < n_rem ? r : n_rem - 1;
            voff_b[t] = (unsigned int)rg * (unsigned int)ldb * ES + (unsigned int)c * 16u;
        } else {
            const int kr = ch * Cfg::B_RPC + lane / Cfg::B_CPR;
            const int c = (lane % Cfg::B_CPR) ^ swz_b<BF16>(kr);
            // likewise column chunks past the end of B.  (When the rows are not whole 16-byte
            // chunks, the row's last, partly filled chunk is read together with the start of the
            // next row, which only feeds output columns that do not exist; at the end of the
            // array the buffer resource cuts it off.)
            constexpr int EPC = 16 / ES;                      // elements per chunk
            const int cg = c * EPC < n_rem ? c : (n_rem + EPC - 1) / EPC - 1;
            voff_b[t] = (unsigned int)kr * (unsigned int)ldb * ES + (unsigned int)cg * 16u;
        }
    }

    auto lds_a = [&](auto st) __attribute__((always_inline)) -> unsigned char* {
        constexpr int v = decltype(st)::value;
        if constexpr (v == 0) return lds_a0; else if constexpr (v == 1) return lds_a1; else return lds_a2;
    };
    auto lds_b = [&](auto st) __attribute__((always_inline)) -> unsigned char* {
        if constexpr (decltype(st)::value == 0) return lds_b0; else return lds_b1;
    };

    // global -> LDS copies of K tile kt: the A part into A stage `st`, the B part into
    // B stage `st`; instruction t of this wave's share (one contiguous 1 KiB of LDS each).
    // Buffer addressing: a scalar resource whose base is this K tile of the workgroup's
    // A (or B) panel, plus the lane's constant 32-bit byte offset -- no vector ALU work
    // per copy.  The resource covers 4 GiB from its base; lane offsets stay below that
    // (checked on the host).
    // `bounded`: the resource ends where the array ends instead of 4 GiB after its base
    // (partial last K tile only; out-of-range lanes then fetch nothing).
    auto records = [](const unsigned char* base, const unsigned char* end, bool bounded) __attribute__((always_inline)) -> int {
        const size_t left = (size_t)(end - base);
        return (bounded && left < 0xffffffffull) ? (int)(unsigned int)left : (int)0xffffffffu;
    };
    // The tiles of A and of B are copied in the order they are processed, each exactly once, so
    // where the next one starts is running state: one step further along K, back to the start
    // of the K range after its last tile (a rotated loop starts at tile k_rot and wraps around).
    size_t a_next_off = (size_t)k_rot * a_step;
    int a_next_tile = k_rot;
    auto copy_a_op = [&](int kt, auto st, int t, bool bounded) __attribute__((always_inline)) {
        (void)kt;
        unsigned char* la = lds_a(st) + wave * (Cfg::A_CPW * 1024);
        const unsigned char* base = Ag + a_next_off;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, records(base, A_end, bounded), 0x00020000),
            PGK_LDS(la + t * 1024), 16, voff_a[t], 0, 0, 0);
        if (t == Cfg::A_CPW - 1) {        // the tile's last piece: move on to the next tile
            a_next_off += a_step;
            if constexpr (VIEW == VIEW_GEMM) {
                if (++a_next_tile == KT) { a_next_tile = 0; a_next_off = 0; }
            }
        }
    };
    // B tiles likewise: b_step further down -- in a convolution's view, after every
    // b_tiles_per_tap tiles the rows start over and the columns move on by b_tap_step elements
    // (a convolution read as a sum of shifted GEMMs, tap after tap).
    // The tap table is handed out from a vector register pair -- lane t holds the entry of tap t --
    // with v_readlane: an index known only at run time into the by-value argument would cost a
    // memory access per tap inside the pinned instruction sequence of the main loop (and its wait
    // would also wait for every LDS fetch in flight).
    long long tap_of_lane = 0;
    if constexpr (VIEW == VIEW_CONV) {
        const __attribute__((address_space(4))) long long* const tap_table =
            (const __attribute__((address_space(4))) long long*)((const __attribute__((address_space(4))) char*)
                __builtin_amdgcn_kernarg_segment_ptr() + offsetof(GemmArgs, b_tap_off));
        tap_of_lane = tap_table[lane & 31];
    }
    auto tap_entry = [&](int t) __attribute__((always_inline)) -> long long {
        const unsigned int lo = (unsigned int)__builtin_amdgcn_readlane((int)(unsigned int)(unsigned long long)tap_of_lane, t);
        const unsigned int hi = (unsigned int)__builtin_amdgcn_readlane((int)(unsigned int)((unsigned long long)tap_of_lane >> 32), t);
        return (long long)(((unsigned long long)hi << 32) | lo);
    };
    size_t b_next_off = VIEW == VIEW_CONV ? (p.b_use_tap_table ? (size_t)p.b_tap_off[0] : 0) : (size_t)k_rot * b_step;
    int b_next_row_tile = 0, b_taps_done = 0, b_next_tile = k_rot;
    const long long b_tap_jump = VIEW == VIEW_CONV ? (long long)p.b_tap_step * ES - (long long)p.b_tiles_per_tap * (long long)b_step : 0;
    auto copy_b_op = [&](int kt, auto st, int t, bool bounded) __attribute__((always_inline)) {
        unsigned char* lb = lds_b(st) + wave * (Cfg::B_CPW * 1024);
        (void)kt;
        const unsigned char* base = Bg + b_next_off;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(
            __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, records(base, B_end, bounded), 0x00020000),
            PGK_LDS(lb + t * 1024), 16, voff_b[t], 0, 0, 0);
        if (t == Cfg::B_CPW - 1) {        // the tile's last piece: move on to the next tile
            b_next_off += b_step;
            if constexpr (VIEW == VIEW_GEMM) {
                if (++b_next_tile == KT) { b_next_tile = 0; b_next_off = 0; }
            } else {
                // (written without branches: a branch here would cut the pinned instruction
                // sequence of the tile into basic blocks)
                const bool new_tap = ++b_next_row_tile == p.b_tiles_per_tap;
                b_next_row_tile = new_tap ? 0 : b_next_row_tile;
                b_taps_done += new_tap ? 1 : 0;
                // (the last advance comes after the final tile: the index is kept inside the table)
                const long long from_table = tap_entry(b_taps_done < 32 ? b_taps_done : 31);
                const long long stepped = (long long)b_next_off + b_tap_jump;
                b_next_off = new_tap ? (size_t)(p.b_use_tap_table ? from_table : stepped) : b_next_off;
            }
        }
    };
    auto copy_a = [&](int kt, auto st) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < Cfg::A_CPW; ++t) copy_a_op(kt, st, t, k_partial && kt == KT - 1);
    };
    auto copy_b = [&](int kt, auto st) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < Cfg::B_CPW; ++t) copy_b_op(kt, st, t, k_partial && kt == KT - 1);
    };
    // The columns of a partial last K tile that do not exist: the copy has put whatever
    // follows the row in memory there (A elements at or beyond k_last, B rows at or beyond
    // k_last).  Each lane clears them in the 16-byte pieces it copied itself -- a whole piece,
    // or the upper elements of the piece that k_last falls into; call after the wait for the
    // copies and before the barrier that publishes the tile.
    auto clear_from = [&](unsigned char* piece, int keep) __attribute__((always_inline)) {   // keep: elements that stay
        constexpr int EPC = 16 / ES;
        auto* q = (__attribute__((address_space(3))) u32x4*)PGK_LDS(piece);
        if (keep <= 0) {
            const u32x4 zero = {0u, 0u, 0u, 0u};
            *q = zero;
        } else if (keep < EPC) {
            u32x4 v = *q;
            const int keep_bytes = keep * ES;
#pragma unroll
            for (int d = 0; d < 4; ++d)
                v[d] &= keep_bytes >= 4 * d + 4 ? 0xffffffffu : keep_bytes <= 4 * d ? 0u : 0x0000ffffu;
            *q = v;
        }
    };
    auto zero_k_tail = [&](auto sta, auto stb) __attribute__((always_inline)) {
        constexpr int EPC = 16 / ES;
#pragma unroll
        for (int t = 0; t < Cfg::A_CPW; ++t) {
            const int r = (wave * Cfg::A_CPW + t) * Cfg::A_RPC + lane / Cfg::A_CPR;
            const int c = (lane % Cfg::A_CPR) ^ swz_a<Cfg::A_CPR>(r);
            clear_from(lds_a(sta) + wave * (Cfg::A_CPW * 1024) + t * 1024 + lane * 16, k_last - c * EPC);
        }
#pragma unroll
        for (int t = 0; t < Cfg::B_CPW; ++t) {
            const int kr = (wave * Cfg::B_CPW + t) * Cfg::B_RPC + lane / Cfg::B_CPR;
            const int cb = (lane % Cfg::B_CPR) ^ swz_a<Cfg::B_CPR>(kr);   // transposed B: kr is a tile column
            clear_from(lds_b(stb) + wave * (Cfg::B_CPW * 1024) + t * 1024 + lane * 16,
                       Cfg::BT ? k_last - cb * EPC : (kr >= k_last ? 0 : EPC));
        }
    };

    // ---- per-lane LDS read offsets
    // fp32 (32 x 32 x 2 instruction): lane = (l32, half); bf16 (16 x 16 x 32): lane = (l16, grp),
    // group grp of sixteen lanes feeds k values 8 grp .. 8 grp + 7 of a step of 32
    const int half = lane >> 5;     // fp32: which K half of the MFMA operand this lane feeds
    const int l32 = lane & 31;
    const int grp = lane >> 4;
    const int l16 = lane & 15;
    constexpr int NKS = BF16 ? BK / 32 : NS;    // steps along K per tile (bf16: of 32; fp32: of 8)
    // A rows (MFMA "B" operand).  fp32: row = wave row base + 32 i + l32, logical chunk 2 s + half;
    // bf16: row = wave row base + 16 i + l16, logical chunk 4 s + grp.  (The swizzle term only
    // depends on the row's low bits, which the block offset leaves alone.)
    int a_koff[NKS];                // per step: row offset + swizzled chunk offset (bytes)
#pragma unroll
    for (int s = 0; s < NKS; ++s) {
        if constexpr (BF16) a_koff[s] = (wm * Cfg::WM + l16) * RA + (((4 * s + grp) ^ swz_a<Cfg::A_CPR>(l16)) * 16);
        else a_koff[s] = (wm * Cfg::WM + l32) * RA + (((2 * s + half) ^ swz_a<Cfg::A_CPR>(l32)) * 16);
    }
    // B columns (MFMA "A" operand)
    constexpr int TNB = BF16 ? Cfg::TN16 : TN;
    int b_off[Cfg::BT ? NKS : TNB];
    if constexpr (Cfg::BT) {
        // transposed B: column n of B is row n of the LDS tile; per step like a_koff
#pragma unroll
        for (int s = 0; s < NKS; ++s) {
            if constexpr (BF16) b_off[s] = (wn * Cfg::WN + l16) * RB + (((4 * s + grp) ^ swz_a<Cfg::B_CPR>(l16)) * 16);
            else b_off[s] = (wn * Cfg::WN + l32) * RB + (((2 * s + half) ^ swz_a<Cfg::B_CPR>(l32)) * 16);
        }
    } else if constexpr (BF16) {
        // a transposing read hands lane i of a sixteen-lane group the four k values of column i:
        // lane pl of the group points at k row pl / 4, columns 4 (pl % 4) ..; group grp reads the
        // rows 8 grp .. of its step (the second half of the eight four rows further down)
        const int pl = lane & 15;
#pragma unroll
        for (int j = 0; j < TNB; ++j) {
            const int n = wn * Cfg::WN + 16 * j + 4 * (pl & 3);
            const int krow = 8 * grp + (pl >> 2);
            const int c = (n >> 3) ^ swz_b<true>(krow);
            b_off[j] = krow * RB + c * 16 + (n & 7) * 2;
        }
    } else {
#pragma unroll
        for (int j = 0; j < TNB; ++j) {
            const int n = wn * Cfg::WN + 32 * j + l32;
            const int krow = 4 * half;
            const int c = (n >> 2) ^ swz_b<false>(krow);
            b_off[j] = krow * RB + c * 16 + (n & 3) * 4;
        }
    }

    // Operand fragments.
    // fp32: one step = 8 K values = four MFMAs per pair of 32 x 32 blocks; fragments of a step in
    // frag[step parity].
    // bf16: one step = one MFMA K (32) for every pair of 16 x 16 blocks, cut into NJH sub-steps over
    // groups of JG B fragments; the A fragments of a step live in fa[step parity], the B fragments
    // of a sub-step in fb[sub-step parity].  A plain B operand arrives as two transposing 64-bit
    // reads per fragment, a transposed one (and A) as one 128-bit read.
    // Below, "step" ss counts sub-steps for bf16: ss = NJH * (step along K) + (fragment group).
    struct FragF32 { f32x4 a[TM]; float b[4][TN]; };
    struct FragF32T { f32x4 a[TM]; f32x4 bt[TN]; };
    struct FragB16 { s16x4 blo[JG], bhi[JG]; };
    struct FragB16T { bf16x8 bt[JG]; };
    using Frag = typename std::conditional<Cfg::BT, typename std::conditional<BF16, FragB16T, FragF32T>::type,
                                           typename std::conditional<BF16, FragB16, FragF32>::type>::type;
    Frag frag[2];
    bf16x8 fa[2][BF16 ? Cfg::TM16 : 1];

    // LDS fetches that step ss needs, numbered in the order its MFMAs need them (the MFMAs run
    // over the A fragments in the outer loop): A fragment 0, every B fragment, then the remaining
    // A fragments.  bf16: the A fragments belong to the first sub-step of a step along K only.
    constexpr int NB_DS = Cfg::BT ? (BF16 ? JG : TN) : BF16 ? 2 * JG : 4 * TN;   // B fetches of a step
    auto n_ds = [](int ss) { return BF16 ? (ss % NJH == 0 ? Cfg::TM16 + NB_DS : NB_DS) : TM + NB_DS; };
    auto fetch_op = [&](auto sta, auto stb, int ss, int q) __attribute__((always_inline)) {
        const unsigned char* as = lds_a(sta);
        const unsigned char* bs = lds_b(stb);
        Frag& f = frag[ss & 1];
        if constexpr (BF16) {
            const int s = ss / NJH, jh = ss % NJH;
            const bool with_a = jh == 0;
            if (with_a && (q == 0 || q > NB_DS)) {
                const int i = q == 0 ? 0 : q - NB_DS;
                fa[s & 1][i] = *(const __attribute__((address_space(3))) bf16x8*)PGK_LDS(as + i * 16 * RA + a_koff[s]);
            } else {
                const int qb = with_a ? q - 1 : q;
                if constexpr (Cfg::BT) {
                    const int j = JG * jh + qb;
                    f.bt[qb] = *(const __attribute__((address_space(3))) bf16x8*)PGK_LDS(bs + j * 16 * RB + b_off[s]);
                } else {
                    const int jj = qb / 2, h = qb % 2;
                    const unsigned char* src = bs + b_off[JG * jh + jj] + (32 * s + 4 * h) * RB;
                    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)PGK_LDS(src));
                    if (h == 0) f.blo[jj] = v; else f.bhi[jj] = v;
                }
            }
        } else {
            const int s = ss;
            if (q == 0 || q > NB_DS) {
                const int i = q == 0 ? 0 : q - NB_DS;
                f.a[i] = *(const __attribute__((address_space(3))) f32x4*)PGK_LDS(as + i * 32 * RA + a_koff[s]);
            } else if constexpr (Cfg::BT) {
                const int j = q - 1;
                f.bt[j] = *(const __attribute__((address_space(3))) f32x4*)PGK_LDS(bs + j * 32 * RB + b_off[s]);
            } else {
                const int t = (q - 1) / TN, j = (q - 1) % TN;
                f.b[t][j] = *(const __attribute__((address_space(3))) float*)PGK_LDS(bs + b_off[j] + (8 * s + t) * RB);
            }
        }
    };
    auto read_frags = [&](auto sta, auto stb, int ss) __attribute__((always_inline)) {
#pragma unroll
        for (int q = 0; q < n_ds(ss); ++q) fetch_op(sta, stb, ss, q);
    };

    // accumulators: fp32 kernels 32 x 32 blocks (acc), bf16 kernels 16 x 16 blocks (acc16)
    f32x16 acc[BF16 ? 1 : TM][BF16 ? 1 : TN];
    f32x4 acc16[BF16 ? Cfg::TM16 : 1][BF16 ? Cfg::TN16 : 1];
    if constexpr (BF16) {
#pragma unroll
        for (int i = 0; i < Cfg::TM16; ++i)
#pragma unroll
            for (int j = 0; j < Cfg::TN16; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc16[i][j][v] = 0.0f;
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    }

    // MFMA number m of step ss (A fragments in the outer loop)
    constexpr int N_MFMA = BF16 ? Cfg::TM16 * JG : 4 * TM * TN;
    auto mfma_op = [&](int ss, int m) __attribute__((always_inline)) {
        const Frag& f = frag[ss & 1];
        if constexpr (BF16) {
            const int s = ss / NJH, jh = ss % NJH;
            const int i = m / JG, jj = m % JG;
            const int j = JG * jh + jj;
            if constexpr (Cfg::BT) {
                acc16[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.bt[jj], fa[s & 1][i], acc16[i][j], 0, 0, 0);
            } else {
                const s16x8 both = __builtin_shufflevector(f.blo[jj], f.bhi[jj], 0, 1, 2, 3, 4, 5, 6, 7);
                acc16[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), fa[s & 1][i], acc16[i][j], 0, 0, 0);
            }
        } else if constexpr (Cfg::BT) {
            const int t = m / (TM * TN), i = (m / TN) % TM, j = m % TN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.bt[j][t], f.a[i][t], acc[i][j], 0, 0, 0);
        } else {
            const int t = m / (TM * TN), i = (m / TN) % TM, j = m % TN;
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.b[t][j], f.a[i][t], acc[i][j], 0, 0, 0);
        }
    };

    // Wait until at most `allowed` of this wave's direct-to-LDS copy instructions are
    // still in flight (they complete in order), and for its own LDS reads; then meet
    // the other waves.  After the barrier the tile that has just landed is visible to
    // everybody, and everybody has fetched its last operands from the stages that are
    // overwritten next.  The sched_barriers keep the compiler from moving MFMAs or
    // fetches across.
    auto wait_copies_and_sync = [&](auto allowed) __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(decltype(allowed)::value) : "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // the same for a partial last K tile landing in stages sta / stb: all copies awaited,
    // missing columns cleared, then the barrier
    auto wait_clear_and_sync = [&](auto sta, auto stb) __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        zero_k_tail(sta, stb);
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // With a three-deep A ring the A copy issued in this tile's first step is for the
    // tile after next and may still be in flight when the next tile is awaited.
    constexpr int STEADY_IN_FLIGHT = (SA - 2) * Cfg::A_CPW;

    // One K tile: A operands from A stage kt % SA, B operands from B stage kt % 2.  ("Step": a
    // sub-step for bf16.)
    //   * Operands of step s+1 are fetched while the MFMAs of step s issue.
    //   * Before the MFMAs of the last step, when a next tile exists: wait for its
    //     copies, meet the other waves, fetch its first operands, and issue the first
    //     half of the copy of tile kt+2 into a stage of this tile, which nobody reads
    //     any more.  The second half follows in the first step of the next tile.
    //   * A rows are 128-byte pieces 2*K bytes apart and take longer to arrive than the
    //     512-byte B rows, so the A half goes first.  Two-deep A ring: A(kt+2) after the
    //     barrier, B(kt+1) in the first step.  Three-deep A ring: A(kt+2) already in
    //     this tile's first step (its stage was last read by tile kt-1), B(kt+2) after
    //     the barrier; the A copy then has a whole extra tile to land.
    //   * Copy instructions are spaced evenly between the MFMAs of their step: a burst
    //     would fill the texture-address path (about 16 cycles per 1 KiB instruction
    //     for the whole CU) and stall the in-order waves (all copies back to back around the
    //     barrier: 9 % more cycles per K tile), while copies in the middle steps of a tile
    //     cost more than in the first and the last one (the A copy spread over three
    //     sub-steps: 3 % more).
    // `steady`: every tile up to kt+SA-1 and kt+2 exists, so the in-flight count at the
    // wait is the steady-state one; otherwise the wait is for all copies.
    // The instruction order of a step is written out and pinned (a scheduling barrier
    // after every MFMA slot): MFMA m, then the operand fetches and copy instructions
    // that belong to slot m, spread evenly over the slots.  The compiler allocates
    // registers and places the lgkmcnt waits; it does not reorder.
    // The fetches go into the first three quarters of the slots, so that the last of
    // them has the remaining MFMAs to come back before the next step needs it.
    // has_a / has_b: tile kt+2 exists (its A / B copy is issued here).
    constexpr int DS_SLOTS = N_MFMA - N_MFMA / 4;
    auto ds_first = [](int m, int nds) { return m >= DS_SLOTS ? nds : (m * nds) / DS_SLOTS; };
    auto tile_body = [&](int kt, auto sta, auto stb, auto steady_tag, bool has_next, bool has_a, bool has_b) __attribute__((always_inline)) {
        constexpr int STA = decltype(sta)::value, STB = decltype(stb)::value;
        constexpr bool STEADY = decltype(steady_tag)::value != 0;
        using NextA = IC<(STA + 1) % SA>;
        using NextB = IC<(STB + 1) % 2>;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const bool last = s + 1 == NS;
            // which copy (if any) is issued during this step
            const bool early = s == 0 && (SA == 3 ? has_a : has_next);    // A(kt+2) or B(kt+1)
            const bool late = last && has_next && (SA == 3 ? has_b : has_a);  // B(kt+2) or A(kt+2)
            const int n_copy = early ? (SA == 3 ? Cfg::A_CPW : Cfg::B_CPW)
                             : late ? (SA == 3 ? Cfg::B_CPW : Cfg::A_CPW) : 0;
            const bool fetch = !last || has_next;
            if (last && has_next) {
                if constexpr (STEADY) {
                    wait_copies_and_sync(IC<STEADY_IN_FLIGHT>{});
                } else {
                    if (k_partial && kt + 2 == KT) wait_clear_and_sync(NextA{}, NextB{});
                    else wait_copies_and_sync(IC<0>{});
                }
            }
            const int nds = n_ds(last ? 0 : s + 1);       // fetches of the step that comes next
#pragma unroll
            for (int m = 0; m < N_MFMA; ++m) {
                mfma_op(s, m);
                if (fetch) {
#pragma unroll
                    for (int q = ds_first(m, nds); q < ds_first(m + 1, nds); ++q) {
                        if (!last) fetch_op(sta, stb, s + 1, q);
                        else fetch_op(NextA{}, NextB{}, 0, q);
                    }
                }
#pragma unroll
                for (int t = 0; t < (Cfg::A_CPW > Cfg::B_CPW ? Cfg::A_CPW : Cfg::B_CPW); ++t) {
                    if (t < (m * n_copy) / N_MFMA || t >= ((m + 1) * n_copy) / N_MFMA) continue;
                    // steady tiles never copy the last K tile when that one is partial
                    const bool b1 = !STEADY && k_partial && kt + 2 == KT, b2 = !STEADY && k_partial && kt + 3 == KT;
                    if constexpr (SA == 3) {
                        if (early) copy_a_op(kt + 2, IC<(STA + 2) % 3>{}, t, b2);
                        else copy_b_op(kt + 2, stb, t, b2);
                    } else {
                        if (early) copy_b_op(kt + 1, NextB{}, t, b1);
                        else copy_a_op(kt + 2, sta, t, b2);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // prologue: tile 0 in full; what a tile body expects to find in flight follows
    copy_a(0, IC<0>{});
    copy_b(0, IC<0>{});
    if constexpr (SA == 3) {
        if (KT > 1) {
            copy_a(1, IC<1>{});
            wait_copies_and_sync(IC<Cfg::A_CPW>{});
            copy_b(1, IC<1>{});
        } else if (k_partial) {
            wait_clear_and_sync(IC<0>{}, IC<0>{});
        } else {
            wait_copies_and_sync(IC<0>{});
        }
    } else {
        if (k_partial && KT == 1) wait_clear_and_sync(IC<0>{}, IC<0>{});
        else wait_copies_and_sync(IC<0>{});
        if (KT > 1) copy_a(1, IC<1>{});
    }
    read_frags(IC<0>{}, IC<0>{}, 0);
    stamp(1);      // the first K tile has landed

    int kt = 0;
    constexpr int UNROLL = SA == 3 ? 6 : 2;      // lcm of the two ring depths
    constexpr int LOOKAHEAD = 2;
    // steady state: every copy issued in the trip exists, no conditionals in the body
    const int KT_full = KT - (k_partial ? 1 : 0);   // the steady loop leaves a partial tile to the tail
    for (; kt + UNROLL - 1 + LOOKAHEAD < KT_full; kt += UNROLL) {
        tile_body(kt, IC<0>{}, IC<0>{}, IC<1>{}, true, true, true);
        tile_body(kt + 1, IC<1 % SA>{}, IC<1>{}, IC<1>{}, true, true, true);
        if constexpr (SA == 3) {
            tile_body(kt + 2, IC<2 % SA>{}, IC<0>{}, IC<1>{}, true, true, true);
            tile_body(kt + 3, IC<3 % SA>{}, IC<1>{}, IC<1>{}, true, true, true);
            tile_body(kt + 4, IC<4 % SA>{}, IC<0>{}, IC<1>{}, true, true, true);
            tile_body(kt + 5, IC<5 % SA>{}, IC<1>{}, IC<1>{}, true, true, true);
        }
    }
    // tail: the remaining tiles (at most UNROLL + LOOKAHEAD), with run-time
    // existence checks and a wait for all copies at each barrier
    auto tail_tile = [&](int t, auto sta, auto stb) __attribute__((always_inline)) {
        if (t < KT) tile_body(t, sta, stb, IC<0>{}, t + 1 < KT, t + 2 < KT, t + 2 < KT);
    };
    tail_tile(kt, IC<0>{}, IC<0>{});
    tail_tile(kt + 1, IC<1 % SA>{}, IC<1>{});
    tail_tile(kt + 2, IC<2 % SA>{}, IC<0>{});
    tail_tile(kt + 3, IC<3 % SA>{}, IC<1>{});
    if constexpr (SA == 3) {
        tail_tile(kt + 4, IC<4 % SA>{}, IC<0>{});
        tail_tile(kt + 5, IC<5 % SA>{}, IC<1>{});
        tail_tile(kt + 6, IC<6 % SA>{}, IC<0>{});
        tail_tile(kt + 7, IC<7 % SA>{}, IC<1>{});
    }

    // ---- epilogue: activation into LDS (the operand buffers are free now), then
    // whole-row stores.  The row-sum exchange has a small buffer of its own.
    // the output tile is staged in pieces of PIECE_BYTES, whole 32-row blocks each, in the two
    // stages of the larger operand and, when it needs more than two pieces, two of the other
    constexpr int OUT_BYTES = BM * BN * (BF16 ? 2 : 4);
    constexpr int OUT_PIECES = (OUT_BYTES + Cfg::PIECE_BYTES - 1) / Cfg::PIECE_BYTES;
    static_assert(OUT_PIECES <= 4 && (OUT_PIECES <= 2 || Cfg::B_BYTES == Cfg::A_BYTES) &&
                  (Cfg::PIECE_BYTES / (BN * (BF16 ? 2 : 4))) % 32 == 0,
                  "the operand buffers hold the output tile, whole 32-row blocks each");
    // (split-K pass 1 of an fp32 kernel stages the same number of bytes; bf16 kernels store
    // their fp32 partial products directly)
    // row-sum exchange buffer: the third A stage when there is one, else a small array
    // (followed by the tile's biases, BIAS_N floats)
    __shared__ __attribute__((aligned(16))) float rs_own[SA > 2 ? 4 : Cfg::WGN * BM + 2 * BIAS_N];
    float* rs_buf = SA > 2 ? (float*)lds_a2 : rs_own;
    static_assert((Cfg::WGN * BM + 2 * BIAS_N) * 4 <= Cfg::A_BYTES, "row-sum and bias buffers fit an A stage");
    unsigned char* const obj[4] = {Cfg::STAGE_IN_B ? lds_b0 : lds_a0, Cfg::STAGE_IN_B ? lds_b1 : lds_a1,
                                   Cfg::STAGE_IN_B ? lds_a0 : lds_b0, Cfg::STAGE_IN_B ? lds_a1 : lds_b1};
    __syncthreads();   // every wave is done with the operand tiles
    stamp(2);          // end of the main loop
    if (out_mode == 1) {
        // split-K pass 1: raw fp32 partial products to the workspace slice
        // (BF16 kernels stage half of the columns at a time: the fp32 tile is twice
        // the size of the operand buffers)
        unsigned char* w = (unsigned char*)(p.ws + ((size_t)b * p.splits + sp) * (size_t)p.M * (size_t)p.N +
                                            (size_t)tm * BM * (size_t)p.N + (size_t)tn * BN);
        if constexpr (!BF16) {
            epilogue_wave32<ACT_NONE, EPI_PLAIN, Cfg, false, false>(acc, nullptr, nullptr, w, (size_t)p.N * 4, m_rem, n_rem,
                                                                    wm, wn, wave, lane, obj, nullptr);
        } else {
#pragma unroll
            for (int i = 0; i < Cfg::TM16; ++i) {
                const int row = wm * Cfg::WM + 16 * i + l16;
                const size_t row_off = (size_t)row * (size_t)p.N;
#pragma unroll
                for (int j = 0; j < Cfg::TN16; ++j) {
                    const int n = wn * Cfg::WN + 16 * j + 4 * grp;
                    const f32x4 o = acc16[i][j];
                    if (row < m_rem) {
                        if (n + 4 <= n_rem) {
                            typedef f32x4 f32x4_at_element __attribute__((aligned(4)));   // rows of any N
                            *(f32x4_at_element*)((float*)w + row_off + n) = o;
                        } else {
#pragma unroll
                            for (int e = 0; e < 3; ++e)
                                if (n + e < n_rem) ((float*)w)[row_off + n + e] = o[e];
                        }
                    }
                }
            }
        }
        return;
    }

    float* rs_lds = p.rs_part ? rs_buf : nullptr;
    // the tile's biases, fetched at kernel start, go through LDS to the lanes that need them
    // (sixteen dependent global loads per lane at this point cost 12 000 cycles per tile)
    float* const bias_lds = rs_buf + Cfg::WGN * BM;
    // (row biases go to a second array; the column array then holds zeros, and so it does
    // when the call has no bias)
    float* const bias_lds_row = bias_lds + BIAS_N;
    if (tid < BIAS_N) {
        bias_lds[tid] = BIAS_PER_ROW ? 0.0f : bias_pre;
        if constexpr (BIAS_PER_ROW) bias_lds_row[tid] = bias_pre;
    }
    __syncthreads();
    const float* const bias_col = bias_lds;
    // Epilogue kinds: plain (column bias only: one add per output), with row sums over a full tile
    // (no masking), with row sums over a ragged last tile column (columns past N masked out), and
    // the convolution's (one bias per row, no row sums).
    unsigned char* c_tile = (unsigned char*)p.C +
        ((size_t)b * p.M * p.N + (size_t)tm * BM * (size_t)p.N + (size_t)tn * BN) * ES;
    // bf16 tiles whose waves own row pieces of at least one 128-byte line stage and store per wave
    // (so do all fp32 tiles: their waves' row pieces are 128 or 256 bytes)
    constexpr bool WAVE_EPILOGUE = !BF16 || Cfg::WN * 2 >= 128;
    stamp(3);          // biases staged (per-wave epilogue: what follows is activation, staging and stores interleaved)
    auto run_epilogue = [&](auto kind) __attribute__((always_inline)) {
        constexpr int KIND = decltype(kind)::value;
        const float* br = KIND == EPI_ROWBIAS ? bias_lds_row : nullptr;
        if constexpr (BF16 && WAVE_EPILOGUE) {
            switch (p.act) {
            case ACT_RELU: epilogue_wave16<ACT_RELU, KIND, Cfg>(acc16, bias_col, br, c_tile, (size_t)p.N * ES, m_rem, n_rem, wm, wn, wave, lane, obj, rs_lds); break;
            case ACT_GELU_TANH: epilogue_wave16<ACT_GELU_TANH, KIND, Cfg>(acc16, bias_col, br, c_tile, (size_t)p.N * ES, m_rem, n_rem, wm, wn, wave, lane, obj, rs_lds); break;
            case ACT_SILU: epilogue_wave16<ACT_SILU, KIND, Cfg>(acc16, bias_col, br, c_tile, (size_t)p.N * ES, m_rem, n_rem, wm, wn, wave, lane, obj, rs_lds); break;
            default: epilogue_wave16<ACT_NONE, KIND, Cfg>(acc16, bias_col, br, c_tile, (size_t)p.N * ES, m_rem, n_rem, wm, wn, wave, lane, obj, rs_lds); break;
            }
        } else if constexpr (BF16) {
            switch (p.act) {
            case ACT_RELU: epilogue_to_lds16<ACT_RELU, KIND, Cfg>(acc16, bias_col, br, n_rem, wm, wn, lane, obj, rs_lds); break;
            case ACT_GELU_TANH: epilogue_to_lds16<ACT_GELU_TANH, KIND, Cfg>(acc16, bias_col, br, n_rem, wm, wn, lane, obj, rs_lds); break;
            case ACT_SILU: epilogue_to_lds16<ACT_SILU, KIND, Cfg>(acc16, bias_col, br, n_rem, wm, wn, lane, obj, rs_lds); break;
            default: epilogue_to_lds16<ACT_NONE, KIND, Cfg>(acc16, bias_col, br, n_rem, wm, wn, lane, obj, rs_lds); break;
            }
        } else {
            switch (p.act) {
            case ACT_RELU: epilogue_wave32<ACT_RELU, KIND, Cfg, true, true>(acc, bias_col, br, c_tile, (size_t)p.N * ES, m_rem, n_rem, wm, wn, wave, lane, obj, rs_lds); break;
            case ACT_GELU_TANH: epilogue_wave32<ACT_GELU_TANH, KIND, Cfg, true, true>(acc, bias_col, br, c_tile, (size_t)p.N * ES, m_rem, n_rem, wm, wn, wave, lane, obj, rs_lds); break;
            case ACT_SILU: epilogue_wave32<ACT_SILU, KIND, Cfg, true, true>(acc, bias_col, br, c_tile, (size_t)p.N * ES, m_rem, n_rem, wm, wn, wave, lane, obj, rs_lds); break;
            default: epilogue_wave32<ACT_NONE, KIND, Cfg, true, true>(acc, bias_col, br, c_tile, (size_t)p.N * ES, m_rem, n_rem, wm, wn, wave, lane, obj, rs_lds); break;
            }
        }
    };
    if constexpr (VIEW == VIEW_CONV) {
        if (p.bias) run_epilogue(IC<EPI_ROWBIAS>{});
        else run_epilogue(IC<EPI_PLAIN>{});
    } else {
        if (!rs_lds) run_epilogue(IC<EPI_PLAIN>{});
        else if (n_rem == BN) run_epilogue(IC<EPI_ROWSUM>{});
        else run_epilogue(IC<EPI_ROWSUM_MASKED>{});
    }
    // (the per-wave epilogue has stored its output already; its waves only meet again when
    // they have row sums to add up)
    if (!WAVE_EPILOGUE || p.rs_part) __syncthreads();
    if constexpr (!WAVE_EPILOGUE) epilogue_store<BF16, Cfg, true>(c_tile, (size_t)p.N * ES, tid, m_rem, n_rem, obj);
    if (p.rs_part && tid < m_rem) {
        // partial row sums of the waves that share a row, added in wave-column order
        float s = rs_buf[tid];
#pragma unroll
        for (int w = 1; w < Cfg::WGN; ++w) s += rs_buf[w * BM + tid];
        p.rs_part[((size_t)b * p.tiles_n + tn) * (size_t)p.M + (size_t)tm * BM + tid] = s;
    }
    stamp(4);          // stores issued
    if constexpr (TIMED) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        stamp(5);      // every wave's stores acknowledged
    }
#endif
}

// Shipping configurations: <bf16, BM, BN, BK, wave rows, wave cols, A ring depth, waves/SIMD>.
// Large tiles for problems that fill the chip with them:
//   bf16 256x256x64, eight waves of 64x128 (two per SIMD, so one wave's operand fetches
//        and barrier waits overlap the other's MFMAs), A ring 3 + B ring 2 = 160 KiB LDS;
//   fp32 128x128x32, four waves of 64x64, 64 KiB of LDS, two workgroups per CU.
// Small tiles (a quarter of the area) for problems whose large-tile grid would leave
// most of the 256 CUs idle:
//   bf16 128x128x64, four waves of 64x64, 80 KiB of LDS, two workgroups per CU;
//   fp32 64x64x32, four waves of 32x32, 32 KiB of LDS.
using CfgBF16 = MfmaCfg<true, 256, 256, 64, 4, 2, 3, 2>;
using CfgF32 = MfmaCfg<false, 128, 128, 32, 2, 2, 2, 1>;
using CfgBF16Small = MfmaCfg<true, 128, 128, 64, 2, 2, 3, 2>;
using CfgF32Small = MfmaCfg<false, 64, 64, 32, 2, 2, 2, 2>;
// Halves of the large bf16 tile, eight waves of 64x64, for outputs whose last tile column (tall,
// 256x128) or last tile row (wide, 128x256) would be at most half full with the large tile:
using CfgBF16Tall = MfmaCfg<true, 256, 128, 64, 4, 2, 3, 2>;
using CfgBF16Wide = MfmaCfg<true, 128, 256, 64, 2, 4, 3, 2>;
// the same four for B given transposed ([N][K])
using CfgBF16T = MfmaCfgBt<true, 256, 256, 64, 4, 2, 3, 2>;
using CfgF32T = MfmaCfgBt<false, 128, 128, 32, 2, 2, 2, 1>;
using CfgBF16SmallT = MfmaCfgBt<true, 128, 128, 64, 2, 2, 3, 2>;
using CfgF32SmallT = MfmaCfgBt<false, 64, 64, 32, 2, 2, 2, 2>;
using CfgBF16TallT = MfmaCfgBt<true, 256, 128, 64, 4, 2, 3, 2>;
using CfgBF16WideT = MfmaCfgBt<true, 128, 256, 64, 2, 4, 3, 2>;
// Skinny tiles, four waves of 32x32, for outputs with at most 32 columns or rows, where the
// tiles above would spend most of their matrix work and LDS traffic on padding and turn a
// memory-bound product into a compute-bound one:
//   narrow 128x32 (B transposed only: a plain B tile would have rows of 64 bytes; the host
//          transposes such a B, which is small), flat 32x128 (either layout of B).
// Two-deep rings, 40 KiB of LDS (fp32 and bf16 alike): these run at the latency of the operand
// stream, and the third A stage bought nothing (bf16 16384 x 16 x 16384: 145 us with it, 137 without).
using CfgBF16NarrowT = MfmaCfgBt<true, 128, 32, 64, 4, 1, 2, 2>;
using CfgF32NarrowT = MfmaCfgBt<false, 128, 32, 32, 4, 1, 2, 2>;
using CfgBF16Flat = MfmaCfg<true, 32, 128, 64, 1, 4, 2, 2>;
using CfgF32Flat = MfmaCfg<false, 32, 128, 32, 1, 4, 2, 2>;
using CfgBF16FlatT = MfmaCfgBt<true, 32, 128, 64, 1, 4, 2, 2>;
using CfgF32FlatT = MfmaCfgBt<false, 32, 128, 32, 1, 4, 2, 2>;

template <typename Cfg, int VIEW, bool TIMED = false>
static hipError_t launch_cfg(const GemmArgs& a, int out_mode, hipStream_t s)
{
    const long long wgs = (long long)a.tiles_m * a.tiles_n * a.batch * a.splits;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    if (TIMED != (a.stamps != nullptr)) return hipErrorInvalidValue;
    hipLaunchKernelGGL((gemm_mfma_kernel<Cfg, VIEW, TIMED>), dim3((unsigned int)wgs), dim3(Cfg::NT), 0, s, a, out_mode);
    return hipGetLastError();
}

}  // namespace pgk
#endif
