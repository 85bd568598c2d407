/*
 * libpgk -- fused GEMM + epilogue kernels for AMD MI355X (CDNA4, gfx950).
 *
 * C ABI: plain pointers and sizes, no C++ or framework types.  Every data
 * pointer below is a DEVICE pointer (HIP global memory on the current device)
 * unless it says otherwise; `stream` is a hipStream_t passed as void*
 * (NULL = the default stream).
 *
 * Operator.  PRAGMA (arXiv 2511.06345) optimises operator kernels -- Section 1
 * names matrix multiplication and reduction operators, Section 4.2 lists the
 * matmul, activation and pooling/reduction categories -- and gives no formula
 * for them, so the operation is the textbook one:
 *
 *     x[b,i,j]    = bias[j] + sum_k A[b,i,k] * B[b,k,j]      (fp32 accumulate)
 *     C[b,i,j]    = act(x[b,i,j])
 *     rowsum[b,i] = sum_j act(x[b,i,j])                      (fp32, taken before
 *                                                             C is rounded to bf16)
 *
 * Layout (all dense, row-major, batch-major):
 *     A      [batch][M][K]   float32, or bfloat16 when dtype = PGK_DTYPE_BF16
 *     B      [batch][K][N]   same element type as A
 *     bias   [N]             float32, shared by every row and batch; NULL = 0
 *     C      [batch][M][N]   same element type as A (bf16: round-to-nearest-even)
 *     rowsum [batch][M]      float32; NULL = row reduction not computed
 *
 * Ownership.  The caller owns every buffer, the workspace included: the library
 * allocates and frees no device memory, keeps no state between calls, and records
 * nothing but kernel launches on `stream` (no memset, no copy node), so every call
 * may be captured into a HIP graph, a first call included.  Outputs are fully
 * overwritten (no accumulate-into-C).  Calls enqueue work on `stream` and return
 * without synchronising it.  Results are deterministic: no value is accumulated
 * with an atomic, every reduction has a fixed order, so equal inputs give bit-equal
 * outputs.
 *
 * Workspace.  Calls that need device memory beyond their inputs and outputs (partial
 * row sums of several tile columns, partial products of a K split, zero-padded copies
 * of operands the matrix-core kernels cannot read in place, segment results of a
 * reduction) take it from `workspace`: device memory of at least the number of bytes
 * the matching *_workspace_bytes query returns, starting on a 16-byte boundary, owned
 * by the caller, contents destroyed by the call, free for reuse once the work the call
 * enqueued has run.  A query that returns 0 means workspace may be NULL.  Too small,
 * misaligned or NULL where bytes are needed gives PGK_ERR_WORKSPACE.  Two calls that
 * may run at the same time (different streams) need different workspaces.
 *
 * Errors.  Every entry point returns a pgk_status_t as int.  Arguments, sizes and
 * the workspace are validated on the host before any device work is enqueued:
 * PGK_ERR_INVALID_ARG, PGK_ERR_UNSUPPORTED and PGK_ERR_WORKSPACE mean that nothing
 * was launched.  PGK_ERR_HIP means the runtime refused a launch; launches of the
 * same call that came before it stay enqueued, and the contents of the outputs and
 * of the workspace are then undefined.
 */
#ifndef PGK_H
#define PGK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PGK_ACT_NONE = 0,      /* y = x */
    PGK_ACT_RELU = 1,      /* y = max(x, 0) */
    PGK_ACT_GELU_TANH = 2, /* y = 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) */
    PGK_ACT_SILU = 3       /* y = x / (1 + exp(-x)) */
} pgk_act_t;

typedef enum {
    PGK_DTYPE_F32 = 0, /* A, B, C float32 */
    PGK_DTYPE_BF16 = 1 /* A, B, C bfloat16; bias, rowsum, accumulation float32 */
} pgk_dtype_t;

typedef enum {
    PGK_OK = 0,
    PGK_ERR_INVALID_ARG = -1, /* NULL A/B/C, non-positive size, unknown act/dtype, bad splits */
    PGK_ERR_UNSUPPORTED = -2, /* size beyond what the kernels index (see each call) */
    PGK_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or smaller than the matching query says */
    PGK_ERR_HIP = -4          /* the HIP runtime refused a launch */
} pgk_status_t;

/* What the workspace queries need to know beyond the sizes (bitwise or). */
typedef enum {
    PGK_WS_ROWSUM = 1,       /* the call is made with rowsum != NULL */
    PGK_WS_B_TRANSPOSED = 2, /* the _bt form of the call (second factor as [batch][N][K]) */
    PGK_WS_UNALIGNED = 4     /* A or B does not start on a 16-byte boundary */
} pgk_ws_flags_t;

/*
 * pgk_gemm_fused -- one launch sequence computing C = act(A*B + bias) and,
 * when rowsum != NULL, rowsum = C*1 (the matmul operator of Sections 1 / 4.2
 * with the activation and reduction operators fused into its epilogue).
 *
 * M, N, K, batch > 0.  Any shape is accepted; M, N and K need not be tile multiples.
 * (Tile shapes: 256 x 256, 128 x 128, 256 x 128, 128 x 256 for bfloat16, 128 x 128 and 64 x 64 for
 * float32, 128 x 32 and 32 x 128 for outputs of at most 32 columns or rows, and 32 x 32 tiles whose
 * waves split the K range for float32 problems of a few tiles and a short K; pgk_gemm_plan tells.)
 * The matrix-core kernels read operands in place when their rows start on 4-byte boundaries
 * (float32 always; bfloat16 when K -- and, for B as [K][N], N -- is even).  Otherwise, when
 * the problem has at least 64^3 multiply-adds, the operands are first copied into the
 * workspace with rows padded with zeros to whole 16-byte chunks (up to batch*(M*K' + K'*N')
 * elements, K' and N' the next multiples of 8).  C, bias and rowsum are always used in place,
 * whatever N is and wherever they start (element alignment).  A B given as [K][N] with at
 * most 32 columns (under an output of more than 32 rows) is likewise copied first, in
 * transposed form, so that the product can run on the 128 x 32 tile, and so is an A or B
 * that does not start on a 16-byte boundary.  What is left for a slower, bounds-checked
 * kernel: problems below 64^3 multiply-adds that would need such a copy, and outputs below
 * 16 x 16 with K below 1024.
 * M, N, K must each be below 2^31 and batch*M*N, batch*M*K, batch*K*N below 2^62 (else
 * PGK_ERR_UNSUPPORTED).
 *
 * workspace: pgk_gemm_fused_workspace_bytes(M, N, K, batch, dtype, flags) bytes (see
 * "Workspace" above); NULL / 0 when that is 0, as it is for problems that fill the chip,
 * have aligned operands and either no row sums or a single tile column.  Besides the operand
 * copies it holds the per-tile-column partial row sums when rowsum is requested and N spans
 * several tile columns (they are added in tile-column order by a second small kernel), and --
 * for problems with few output tiles and a long K (a grid that would leave most of the chip
 * idle -- fewer than 192 tiles of the shape in use, 384 for the skinny tiles -- and K long
 * enough for at least two slices; or fewer than 192 large tiles and K of at least 512 K
 * tiles; pgk_gemm_plan tells) -- the partial products of an automatic K split, computed
 * exactly as by pgk_gemm_splitk with splits = 0 (at most 256 MiB; larger cases are not
 * split).  Which route a problem takes depends on its shape and on the alignment of A and B
 * only, so results stay bit-reproducible.
 */
int pgk_gemm_fused(const void* A, const void* B, const float* bias, void* C, float* rowsum,
                   int64_t M, int64_t N, int64_t K, int64_t batch,
                   int act, int dtype,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace pgk_gemm_fused (or, with PGK_WS_B_TRANSPOSED, pgk_gemm_fused_bt) needs
 * for this problem; `flags` is a bitwise or of pgk_ws_flags_t saying how the call will be
 * made.  Pure host arithmetic; 0 also for invalid arguments (the call then reports them). */
size_t pgk_gemm_fused_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int flags);

/*
 * pgk_gemm_fused_static -- pgk_gemm_fused for callers that cannot hand over a workspace and
 * cannot allocate one either (code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation): same operator, same kernels, same results bit for bit, with the
 * workspace taken from a fixed array of pgk_gemm_fused_static_max_bytes() = 4 MiB that is part
 * of the library's device image (every GPU the library runs on holds one copy until the process
 * ends).  The call allocates nothing and frees nothing.  `stream` must belong to the current
 * device.  A problem whose pgk_gemm_fused_workspace_bytes exceeds the array (a large automatic
 * K split, large operand copies) gets PGK_ERR_WORKSPACE: nothing is launched, use pgk_gemm_fused.
 * All calls on one GPU share that GPU's array, which is left holding the last call's partial
 * results: two calls that may run at the same time on one GPU (different streams) race and give
 * undefined results -- order them, or use pgk_gemm_fused with a workspace each.
 */
int pgk_gemm_fused_static(const void* A, const void* B, const float* bias, void* C, float* rowsum,
                          int64_t M, int64_t N, int64_t K, int64_t batch,
                          int act, int dtype, void* stream);
size_t pgk_gemm_fused_static_max_bytes(void);

/*
 * pgk_gemm_splitk -- the same operator for small M,N and large K, computed in
 * two passes so that enough workgroups exist to fill the chip:
 *   pass 1: split s of `splits` multiplies a contiguous K-slice and stores its
 *           raw fp32 partial product to workspace[b][s][M][N];
 *   pass 2: per output element, partials are added in the order s = 0, 1, ...,
 *           then bias, activation, store, and the row sum in a fixed order.
 * The result is bit-reproducible for given inputs and `splits`.
 *
 * splits >= 1, or 0 to let the library choose (pgk_splitk_auto_splits): the smallest
 * number of slices that fills the chip with the tile shape chosen with it (256 workgroups
 * of the large bfloat16 tile, 1024 of the small float32 tile, else 512), with slices of
 * at least 16 K tiles (32 for bfloat16 outputs of 96 and more 128 x 128 tiles) and at most
 * 32 slices.  The
 * K range is cut into slices of L = kstep * ceil(ceil(K / kstep) / splits)
 * elements (kstep = the kernel's K tile: 32 for float32, 64 for bfloat16);
 * slice s covers [s*L, min(K, (s+1)*L)); trailing empty slices are dropped.
 * splits > K is PGK_ERR_INVALID_ARG.
 *
 * workspace: device buffer of at least pgk_splitk_workspace_bytes(...) bytes (or the exact
 * pgk_gemm_splitk_workspace_bytes(..., flags)), 16-byte aligned, owned by the caller,
 * contents destroyed: the partial products first, then the per-segment partial row sums
 * of a skinny output's second pass and the operand copies described under pgk_gemm_fused,
 * where the problem has them.  Too small or NULL gives PGK_ERR_WORKSPACE.
 */
int pgk_gemm_splitk(const void* A, const void* B, const float* bias, void* C, float* rowsum,
                    int64_t M, int64_t N, int64_t K, int64_t batch,
                    int act, int dtype, int splits,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * pgk_gemm_fused_bt / pgk_gemm_splitk_bt -- the same two calls with the second factor
 * given transposed: Bt [batch][N][K], K contiguous (how a linear layer's weight
 * [out_features][in_features] is stored), so that C = act(A * Bt^T + bias).  This is the
 * "pre-transposed B" form of the matmul operator (Sections 1 / 4.2; same definition, only
 * the storage of one operand differs).  Every other argument, the layouts of A, bias, C
 * and rowsum, ownership, the workspace, the split rule and the errors are as for
 * pgk_gemm_fused / pgk_gemm_splitk (workspace queries: flag PGK_WS_B_TRANSPOSED;
 * pgk_splitk_workspace_bytes covers both layouts).  The matrix-core kernels read Bt in place -- no
 * transposed copy is made -- when its rows start on 4-byte boundaries (float32, or an even
 * K), whatever N is; otherwise A and Bt are copied with K padded, as described there.
 */
int pgk_gemm_fused_bt(const void* A, const void* Bt, const float* bias, void* C, float* rowsum,
                      int64_t M, int64_t N, int64_t K, int64_t batch,
                      int act, int dtype,
                      void* workspace, size_t workspace_bytes, void* stream);
int pgk_gemm_splitk_bt(const void* A, const void* Bt, const float* bias, void* C, float* rowsum,
                       int64_t M, int64_t N, int64_t K, int64_t batch,
                       int act, int dtype, int splits,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * pgk_gemm_plan -- what pgk_gemm_fused (b_transposed = 0) or pgk_gemm_fused_bt (1) runs for a
 * problem whose pointers are all 16-byte aligned: the tile-shape table and the split rule as a
 * pure host function, for callers that want to know and for tests (the paper, Section 4.2, credits
 * its matmul gains to tile candidates chosen from profile data; this is the static form of such
 * a table).  `out` is a HOST array of six int32:
 *   out[0]  1 = matrix-core kernel, 0 = bounds-checked kernel
 *   out[1..3]  tile rows, tile columns, K tile
 *   out[4]  K slices (1 = one pass; more = the automatic two-pass split)
 *   out[5]  workgroups of the GEMM launch
 * Returns PGK_OK, or the error pgk_gemm_fused would return for these sizes; out == NULL is
 * PGK_ERR_INVALID_ARG.  Nothing is launched.
 */
int pgk_gemm_plan(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int b_transposed, int32_t* out);

/* Bytes of workspace that are enough for pgk_gemm_splitk and pgk_gemm_splitk_bt on this
 * problem (splits = 0: the automatic choice), with or without row sums, when A and B start
 * on 16-byte boundaries.  Pure host arithmetic; returns 0 for invalid arguments. */
size_t pgk_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch,
                                  int dtype, int splits);

/* The exact need of one way of making the call (`flags`: bitwise or of pgk_ws_flags_t),
 * operands off the 16-byte grid included.  Never more than pgk_splitk_workspace_bytes
 * unless PGK_WS_UNALIGNED is set.  0 for invalid arguments. */
size_t pgk_gemm_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch,
                                       int dtype, int splits, int flags);

/* The number of splits pgk_gemm_splitk uses for splits = 0, or the effective
 * number (after dropping empty slices) for splits >= 1.  0 for invalid
 * arguments.  Pure host arithmetic. */
int pgk_splitk_auto_splits(int64_t M, int64_t N, int64_t K, int64_t batch,
                           int dtype, int splits);

/*
 * pgk_reduce_max -- maximum over one dimension (the reduction operator of the
 * paper's GPU case study, Section 4.4; no formula is given there, so this is the
 * plain definition).  X is a dense row-major tensor viewed as [outer][red][inner]
 * -- reducing dimension d of a contiguous tensor means outer = product of the sizes
 * before d, red = size of d, inner = product of the sizes after d:
 *
 *     out[o][i] = max over r of X[o][r][i]
 *     idx[o][i] = the smallest r with X[o][r][i] == out[o][i]
 *
 * under IEEE comparison (+0 and -0 tie; the earlier one is returned, bit for bit).
 * A slice that holds a NaN gives that NaN and the position of the first NaN.
 *
 *     X    [outer][red][inner]  float32 or bfloat16 (dtype), device pointer
 *     out  [outer][inner]       same element type as X, device pointer
 *     idx  [outer][inner]       int32 device pointer, or NULL = positions not wanted
 *
 * outer, red, inner > 0; red at most 2^31 - 1024, outer * inner below 2^62, else
 * PGK_ERR_UNSUPPORTED.  Any shape and alignment is accepted (16-byte loads are used when
 * X is 16-byte aligned and the contiguous extent is a multiple of 16 bytes).  When there
 * are few outputs and a long reduced dimension the range is reduced in segments and a
 * second small kernel combines them; the segment results (value, position) live in
 * `workspace`: pgk_reduce_max_workspace_bytes(...) bytes of device memory on a 4-byte
 * boundary, NULL / 0 when that is 0 (see "Workspace" at the top).
 * The result does not depend on how the work was split and is bit-reproducible.
 */
int pgk_reduce_max(const void* X, void* out, int32_t* idx,
                   int64_t outer, int64_t red, int64_t inner, int dtype,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace pgk_reduce_max needs for this shape (enough wherever X starts).  Pure
 * host arithmetic; 0 also for invalid arguments. */
size_t pgk_reduce_max_workspace_bytes(int64_t outer, int64_t red, int64_t inner, int dtype);

/*
 * pgk_conv1d -- one-dimensional convolution with fused bias and activation (the paper's second
 * case study, Section 4.4 "Conv Standard 1D"; no formula is given there, so this is the
 * operator as deep-learning frameworks define it: cross-correlation with zero padding):
 *
 *     y[b][co][l] = act( bias[co] + sum_ci sum_k w[co][ci][k] * x[b][ci][l*stride + k*dilation - pad] )
 *     Lout = floor((L + 2 pad - dilation (Kw - 1) - 1) / stride) + 1      (x outside [0, L) is 0)
 *
 *     x    [B][Cin][L]       float32 or bfloat16 (dtype), device pointer
 *     w    [Cout][Cin][Kw]   same element type
 *     bias [Cout]            float32, NULL = 0
 *     y    [B][Cout][Lout]   same element type as x (bf16: round-to-nearest-even), fully overwritten
 *
 * Accumulation is float32.  Every size > 0, stride, dilation >= 1, pad >= 0, Lout >= 1, sizes
 * within the index ranges of pgk_gemm_fused (else PGK_ERR_INVALID_ARG / PGK_ERR_UNSUPPORTED).
 *
 * The convolution runs on the matrix cores as a sum over the taps of GEMMs on shifted views of
 * the input (no unfolded copy of the input is made) when Lout is at least 16, in one of two
 * ways (where the kernels read x itself, x must start on a 16-byte boundary; w, bias and y may
 * start on any element).
 * Stride 1, Cin a multiple of the K tile (32 float32 / 64 bfloat16) and, for bfloat16, an even
 * dilation (or Kw = 1): the views are taken of the input itself -- only the tile columns at the
 * ends of the rows read small zero-padded strips -- or (also whenever Lout is not a multiple of
 * 16 bytes of elements) of one zero-padded copy of it.  Otherwise
 * -- stride > 1, any Cin of at least half a K tile's multiple (Cin >= its round-up / 2), odd
 * dilation in bfloat16 -- with Kw <= 32: the views are taken of copies of the input, one per
 * phase of the stride (and a second one shifted by one element for bfloat16 taps at odd
 * offsets), channels padded with zeros to a multiple of the K tile.  Both need `workspace`
 * (device memory, 256-byte aligned, contents destroyed) of pgk_conv1d_workspace_bytes(...)
 * bytes for the regrouped weights and the strips or copies.  Too small or NULL gives
 * PGK_ERR_WORKSPACE.  Every other case (a few input channels, tiny outputs) is computed by
 * a bounds-checked kernel that reads the input in place and needs no workspace (the query
 * then returns 0).
 */
int pgk_conv1d(const void* x, const void* w, const float* bias, void* y,
               int64_t B, int64_t Cin, int64_t L, int64_t Cout, int64_t Kw,
               int64_t stride, int64_t pad, int64_t dilation, int act, int dtype,
               void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace pgk_conv1d needs for this problem (0: none).  Pure host arithmetic,
 * assuming 16-byte aligned pointers; 0 also for invalid arguments. */
size_t pgk_conv1d_workspace_bytes(int64_t B, int64_t Cin, int64_t L, int64_t Cout, int64_t Kw,
                                  int64_t stride, int64_t pad, int64_t dilation, int dtype);

/* Output length of the convolution, or 0 when the arguments give none.  Host arithmetic. */
int64_t pgk_conv1d_out_len(int64_t L, int64_t Kw, int64_t stride, int64_t pad, int64_t dilation);

/*
 * pgk_probe_mfma / pgk_probe_mfma_fed / pgk_probe_stream_read / pgk_probe_gemm_phases -- measurement aids, not operators: what the chip
 * sustains under its power limit, to read a kernel's numbers against (the paper's Section 3.2
 * lists matrix-unit activity and memory throughput among a performance engineer's evidence).
 *
 * pgk_probe_mfma launches 512 workgroups (two per CU, two waves per SIMD) in which every wave
 * issues, per iteration, the matrix instructions of `dtype` that the kernels use (bfloat16: 64 of
 * 16 x 16 x 32; float32: 32 of 32 x 32 x 2) on register operands -- all zero
 * (random_operands = 0: nothing toggles, the clock stays high) or random finite values
 * (random_operands = 1: what a real GEMM's operands do to the clock).  *flops_out (host
 * pointer, may be NULL) receives the floating-point operations of one launch.
 * pgk_probe_stream_read reads `bytes` (a multiple of 16, 16-byte aligned device memory at
 * `src`) once with 16-byte loads.  `sink` is one float of device memory for both; it is not
 * written in practice.  Time the calls with events on `stream`.  iters in [1, 2^20].
 */
int pgk_probe_mfma(int dtype, int random_operands, int iters, float* sink, double* flops_out, void* stream);

/*
 * pgk_probe_mfma_fed -- the bfloat16 matrix instruction fed the way the 256 x 256 x 64 GEMM kernel
 * feeds it, and nothing else of that kernel: 256 workgroups of eight waves; per iteration (one
 * "K tile") a wave issues 64 instructions (16 x 16 x 32) whose operands it re-reads from LDS at the
 * kernel's addresses (192 KiB per CU and iteration), all waves meet at one barrier, and with copies != 0
 * the workgroup also copies one 64 KiB piece of `src` straight into LDS (eight 1 KiB
 * instructions per wave), awaited before the barrier.  Read against pgk_probe_mfma with random
 * operands (registers only) it shows what the LDS reads and the copies cost in sustained rate and
 * shader clock under the power limit.
 *
 *     iters           even, in [2, 2^20]
 *     src             device memory, 16-byte aligned, src_bytes a multiple of 64 KiB, holding finite
 *                     bfloat16 values (they become operands); ignored when copies == 0
 *     resident_bytes  multiple of 64 KiB, <= src_bytes: the leading pieces every workgroup cycles
 *                     through (they stay in L2)
 *     stream_every    0, or n > 0: every n-th iteration's piece comes from the rest of src
 *                     instead, each piece read once per launch as long as the rest is large
 *                     enough (a stream from memory, as for operand panels that have left L2)
 *     clock_out       device memory, 8-byte aligned, 3 uint64: [0] shader-clock cycles and [1]
 *                     100 MHz ticks that workgroup 0 spent in its loop; [2] not written in practice
 *     *flops_out      (host pointer, may be NULL) floating-point operations of one launch
 */
int pgk_probe_mfma_fed(int copies, int iters, const void* src, size_t src_bytes, size_t resident_bytes,
                       int stream_every, uint64_t* clock_out, double* flops_out, void* stream);

/*
 * pgk_probe_gemm_phases -- where the time of the large-tile matrix-core kernel goes (the per-phase
 * evidence a performance engineer asks a profiler for, Section 3.2, which the counters do not
 * give): one launch of a measurement instance of the 256 x 256 x 64 bfloat16 kernel or of the
 * 128 x 128 x 32 float32 kernel (`dtype`) on C = act(A*B + bias), batch 1, B as [K][N], in which
 * wave 0 of every workgroup stamps the shader-clock cycle counter and the constant 100 MHz counter
 * at six points -- kernel entry, first K tile landed, end of the main loop, the tile's biases
 * handed out through LDS, output done (bias, activation, row sums, staging through LDS and the
 * stores issued), stores acknowledged.  The instance is the
 * shipping kernel plus those stamps and one wait for the stores at the very end; results in C
 * are the same.
 *
 *     stamps  device memory, 8-byte aligned, 16 uint64 per workgroup (= per output tile, in
 *             launch order): words 2k, 2k+1 = cycles, ticks of stamp k (k = 0..5); word 12 the
 *             hardware id register of the wave, word 13 the XCD number; 14, 15 unused
 *     rowsum_partials  NULL, or device memory for (tile columns) * M floats: the per-tile-column
 *             partial row sums (the row-sum epilogue is then the one timed)
 *     *workgroups_out (host pointer, may be NULL) receives the number of workgroups
 *
 * A and B 16-byte aligned, operand rows on 4-byte boundaries (bfloat16: K and N even); else
 * PGK_ERR_UNSUPPORTED.  stamps_bytes too small: PGK_ERR_WORKSPACE.
 */
int pgk_probe_gemm_phases(const void* A, const void* B, const float* bias, void* C, float* rowsum_partials,
                          int64_t M, int64_t N, int64_t K, int act, int dtype,
                          uint64_t* stamps, size_t stamps_bytes, int32_t* workgroups_out, void* stream);
int pgk_probe_stream_read(const void* src, size_t bytes, float* sink, void* stream);

/* Human-readable name of a status code; never NULL.  Host pointer, static storage. */
const char* pgk_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int pgk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PGK_H */
