// Internal launcher interface between the C-ABI layer and the HIP kernels.
// Not installed; the public contract is include/pgk.h.
#ifndef PGK_KERNELS_H
#define PGK_KERNELS_H

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pgk {

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU_TANH = 2, ACT_SILU = 3 };
enum { DT_F32 = 0, DT_BF16 = 1 };

// One GEMM launch.  Pointers are device pointers.  `out_mode`:
//   0 = fused epilogue: bias + activation, store C, optional row-sum partials
//   1 = split-K pass 1: store the raw fp32 accumulators to `ws`
struct GemmArgs {
    const void* A;      // [batch][M][K]
    const void* B;      // [batch][K][N]
    const float* bias;  // [N] or nullptr
    void* C;            // [batch][M][N]
    float* rs_part;     // row-sum partials [batch][tiles_n][M], or final [batch][M]
                        // when tiles_n == 1; nullptr = no row-sum
    float* ws;          // split-K partial products [batch][splits][M][N]
    int M, N, K, batch;
    // Operand views.  Plain GEMM: a_batch_stride = M*K, b_batch_stride = K*N, ldb = N,
    // b_tiles_per_tap = INT_MAX (fill_plain_views sets these).  a_batch_stride = 0 shares A
    // between the batch entries.
    long long a_batch_stride, b_batch_stride;   // elements between batch entries of A and of B
    int ldb;                 // elements between rows of B
    int b_trans;             // 1: B is given transposed, [batch][N][ldb >= K], K contiguous
    int k_rotate;            // 1: each workgroup starts its K loop at a tile of its own (plain GEMM views, whole K tiles only)
    int b_tail_bounded;      // 1: rows of a plain B are not whole 16-byte chunks: the copies of the last K tile stop at the end of B
    int bias_per_row;        // 0: bias[N] added to columns; 1: bias[M] added to rows (a convolution's views: the
                             // matrix-core kernels then run their convolution instances)
    // Matrix-core kernels, convolution as a sum of shifted GEMMs: K tile kt reads B rows
    // (kt % b_tiles_per_tap) * bk ... at column offset (kt / b_tiles_per_tap) * b_tap_step.
    int b_tiles_per_tap, b_tap_step;
    // ... or, with b_use_tap_table, tap t starts at byte offset b_tap_off[t] from the B base: the
    // taps of a convolution may then read different copies of the input (the phases of a strided
    // convolution; for bf16 a copy shifted by one element for taps at odd column offsets, so
    // that every tile base stays 4-byte aligned).  At most kMaxTableTaps taps.
    int b_use_tap_table;
    long long b_tap_off[32];
    // Matrix-core kernels, convolution without a padded copy of the input: the columns a tile
    // reads start b_col_shift (= -pad) before its output columns; the (at most three) tile
    // columns whose reads would leave the rows read a small zero-padded strip instead:
    // edge_B[e] [batch][rows][edge_ldb], holding the columns of tile column edge_tn[e].
    int b_col_shift;
    const void* edge_B[3];
    int edge_tn[3];
    int edge_ldb;
    long long edge_batch_stride;
    // Bounds-checked kernel, convolution read in place: conv_kw > 0 means B is the input
    // x [batch][K / conv_kw][conv_len] and B[k][n] stands for
    // x[k / conv_kw][n * conv_stride + (k % conv_kw) * conv_dil - conv_pad], zero outside.
    int conv_kw, conv_stride, conv_pad, conv_dil, conv_len;
    int act;
    int splits;         // >= 1
    int k_slice;        // K elements per split (multiple of the K tile)
    int tiles_m, tiles_n;
    int group_m;        // tile rows per scheduling group
    // measurement instance only (launch_gemm_mfma_timed): kStampWords 64-bit words per workgroup
    unsigned long long* stamps;
};

// Words per workgroup the timed instance writes: six (cycle counter, 100 MHz counter) pairs --
// kernel entry, first K tile landed, end of the main loop, biases staged, stores issued,
// stores acknowledged -- then the hardware id register and the XCD number, two words unused.
constexpr int kStampWords = 16;

inline void fill_plain_views(GemmArgs& a)
{
    a.a_batch_stride = (long long)a.M * a.K;
    a.b_batch_stride = (long long)a.K * a.N;
    a.ldb = a.N;
    a.b_trans = 0;
    a.b_tail_bounded = 0;
    a.k_rotate = 0;
    a.bias_per_row = 0;
    a.b_tiles_per_tap = 0x7fffffff;
    a.b_tap_step = 0;
    a.b_use_tap_table = 0;
    for (int t = 0; t < 32; ++t) a.b_tap_off[t] = 0;
    a.b_col_shift = 0;
    for (int e = 0; e < 3; ++e) { a.edge_B[e] = nullptr; a.edge_tn[e] = -1; }
    a.edge_ldb = 0;
    a.edge_batch_stride = 0;
    a.conv_kw = 0; a.conv_stride = 1; a.conv_pad = 0; a.conv_dil = 1; a.conv_len = 0;
}

// B given as [batch][N][K] (call after fill_plain_views)
inline void set_b_transposed(GemmArgs& a)
{
    a.b_trans = 1;
    a.ldb = a.K;
}

// Tile geometry of the matrix-core kernels: a large and a small tile per element type (same
// K tile), the small one for grids that would not fill the chip; for bf16 also the two halves
// of the large tile (tall = half as wide, wide = half as high) for outputs whose last tile
// column / row would be at most half full; and two skinny tiles per type, narrow (32 columns; B
// transposed only) and flat (32 rows).  A kind the type does not have gives the large tile.
struct TileShape { int bm, bn, bk; };
// TILE_TINY (fp32, B as [K][N] only): 32 x 32 tiles whose four waves split the K range -- the
// latency-bound problems of a few tiles (pgk_gemm_tiny.hip).
enum { TILE_LARGE = 0, TILE_SMALL = 1, TILE_TALL = 2, TILE_WIDE = 3, TILE_NARROW = 4, TILE_FLAT = 5, TILE_TINY = 6 };
TileShape mfma_tile_shape(int dtype, int kind);
bool mfma_has_tile(int dtype, int kind, bool b_trans);
TileShape guarded_tile_shape();

// Matrix-core kernels: require k_slice % bk == 0, K and N multiples of the 16-byte
// chunk (8 bf16 / 4 fp32 elements) and 16-byte aligned A, B, C, bias, ws.
// M, N and K need not be tile multiples: edge tiles re-read valid rows / columns and
// store only what exists; the missing columns of a partial last K tile are cleared in LDS.
hipError_t launch_gemm_mfma(const GemmArgs& a, int dtype, int kind, int out_mode, hipStream_t s);
// The instances for a convolution's operand views (bias_per_row = 1, A shared by the batch
// entries, B tiles walking tap after tap, edge strips; B as [K][N], out_mode 0); reached through
// launch_gemm_mfma.
hipError_t launch_gemm_mfma_conv(const GemmArgs& a, int dtype, int kind, int out_mode, hipStream_t s);

// fp32, 32 x 32 tiles, K split over the four waves of a workgroup (out_mode 0; K, N, ldb multiples
// of 4, A and B on 16-byte boundaries); reached through launch_gemm_mfma with TILE_TINY.
TileShape tiny_tile_shape();
hipError_t launch_gemm_tiny(const GemmArgs& a, hipStream_t s);

// The large tile of either type, plain operand views, out_mode 0, with phase stamps (a.stamps set).
hipError_t launch_gemm_mfma_timed(const GemmArgs& a, int dtype, hipStream_t s);

// Bounds-checked kernel for every other shape.
hipError_t launch_gemm_guarded(const GemmArgs& a, int dtype, int out_mode, hipStream_t s);

// rowsum[b][m] = sum over t = 0..tiles_n-1 (in that order) of part[b][t][m]
hipError_t launch_rowsum_combine(const float* part, float* rowsum, int M, int batch,
                                 int tiles_n, hipStream_t s);

// Split-K pass 2: C = act(sum_s ws[b][s] + bias), s ascending; optional rowsum.  The columns
// are cut into `nseg` segments (splitk_reduce_segments) so that skinny outputs still fill the
// chip; with nseg > 1 the row sums go to rs_part[batch][nseg][M] and are to be added in
// segment order (launch_rowsum_combine with tiles_n = nseg).
int splitk_reduce_segments(int M, int N, int batch);
hipError_t launch_splitk_reduce(const float* ws, const float* bias, void* C, float* rowsum, float* rs_part,
                                int nseg, int M, int N, int batch, int splits, int act, int dtype, hipStream_t s);

// Maximum over the middle dimension of X viewed as [outer][red][inner]; see
// pgk_reduce_max.hip.  The plan is pure host arithmetic: vector width (elements per
// 16-byte load, or 1 for the unaligned fallback), lanes per row (inner == 1), number of
// segments the reduced range is cut into and their length (in chunks for inner == 1, in
// r otherwise), workgroups, and the number of (value, position) partials for the second
// pass (0 when there is a single segment).
struct ReducePlan {
    int vec, group, segs, per_seg, tiles_i;
    long long blocks;
    size_t partial_elems;
};
ReducePlan plan_reduce_max(long long outer, long long red, long long inner, int dtype, bool x_aligned);
// pv / pi: partial_elems floats / ints of scratch (unused when partial_elems == 0).
hipError_t launch_reduce_max(const ReducePlan& pl, const void* X, void* out, int* idx, float* pv, int* pi,
                             long long outer, long long red, long long inner, int dtype, hipStream_t s);

// Convolution helpers (pgk_conv.hip): xp[row][j] = x[row][j - pad] inside [0, L), else 0, for
// `rows` rows of length L -> Lp; wr[co][k][ci] = w[co][ci][k].
hipError_t launch_conv_pad_input(const void* x, void* xp, long long rows, int L, int Lp, int pad, int dtype, hipStream_t s);
// Copies of the input for the table-driven path: copy c = phase * shifts + h (phase < stride,
// h < shifts) is xc[c][b][ci][j] = x[b][ci][(j + h) * stride + phase - pad] inside [0, L) and for
// ci < Cin, else 0; ci runs to Cin_pad, j to Lq.
// (the same launch regroups the weights: wr[co][k][ci] = w[co][ci][k], zero up to Cin_pad)
hipError_t launch_conv_phase_copies(const void* x, void* xc, long long B, int Cin, int Cin_pad, int L, int Lq, int pad,
                                    int stride, int shifts, const void* w, void* wr, int Cout, int Kw, int dtype, hipStream_t s);
// wr[co][k][ci] = w[co][ci][k] for ci < Cin, 0 for Cin <= ci < Cin_pad
hipError_t launch_conv_repack_weights(const void* w, void* wr, int Cout, int Cin, int Cin_pad, int Kw, int dtype, hipStream_t s);
// the regrouped weights and, in the same launch, strip e (e < n_edges, may be 0) of
// S[e][row][j], j < W: x[row][first_col[e] + j] inside [0, L), else 0
hipError_t launch_conv_prepare(const void* x, void* strips, long long rows, int L, int W, int n_edges, const int* first_col,
                               const void* w, void* wr, int Cout, int Cin, int Kw, int dtype, hipStream_t s);
constexpr int kMaxTableTaps = 32;

// Operand packing (pgk_pack.hip): dst[b][r][c] = src[b][r][c] inside the source, else 0 (dst rows of
// cols_dst elements, a multiple of the 16-byte chunk).
hipError_t launch_pad_matrix(const void* src, void* dst, long long batch, int rows_src, int cols_src, int rows_dst,
                             int cols_dst, int dtype, hipStream_t s);
// dst[b][n][k] = src[b][k][n] for k < K, 0 up to Kd (a multiple of the chunk): a narrow B transposed
hipError_t launch_transpose_pad(const void* src, void* dst, long long batch, int K, int N, int Kd, int dtype, hipStream_t s);

// Measurement aids (pgk_probe.hip): a matrix-instruction-only loop (workgroups of 256
// threads, `iters` x 32 instructions per wave, zero or random operands) and a streaming
// read of `bytes` (16-byte aligned).  `sink`: one float the kernels never really write.
hipError_t launch_probe_mfma(int dtype, int random_operands, int iters, int workgroups, float* sink, hipStream_t s);
// bf16 matrix instructions with operands re-read from LDS (and, with `copies`, 64 KiB direct-to-LDS
// copies per 32 instructions of a wave): 256 workgroups of 512 threads.  iters even, >= 2;
// src = (resident + streamed) pieces of 64 KiB; clock_out = 3 words of device memory.
hipError_t launch_probe_mfma_fed(bool copies, int iters, const void* src, unsigned int resident, unsigned int streamed,
                                 int stream_every, unsigned long long* clock_out, hipStream_t s);
hipError_t launch_probe_stream_read(const void* src, size_t bytes, float* sink, hipStream_t s);

}  // namespace pgk
#endif
