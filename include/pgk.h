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
 * Ownership.  The caller owns every buffer.  Outputs are fully overwritten
 * (no accumulate-into-C).  Calls enqueue work on `stream` and return without
 * synchronising it.  Results are deterministic: no value is accumulated with an
 * atomic, every reduction has a fixed order, so equal inputs give bit-equal outputs.
 *
 * Errors.  Every entry point returns a pgk_status_t as int.  Arguments are
 * validated on the host before any device work is enqueued, so an error return
 * means nothing was launched.
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
    PGK_ERR_WORKSPACE = -3,   /* workspace missing or smaller than pgk_splitk_workspace_bytes */
    PGK_ERR_HIP = -4          /* the HIP runtime refused a launch or an allocation */
} pgk_status_t;

/*
 * pgk_gemm_fused -- one launch sequence computing C = act(A*B + bias) and,
 * when rowsum != NULL, rowsum = C*1 (the matmul operator of Sections 1 / 4.2
 * with the activation and reduction operators fused into its epilogue).
 *
 * M, N, K, batch > 0.  Any shape is accepted; M, N and K need not be tile multiples.
 * The matrix-core kernels read operands in place when their rows start on 4-byte boundaries
 * (float32 always; bfloat16 when K -- and, for B as [K][N], N -- is even).  Otherwise the
 * operands are first copied into buffers of the library with rows padded with zeros to
 * whole 16-byte chunks (a second per-(device, stream) pool of up to batch*(M*K' + K'*N')
 * elements, K' and N' the next multiples of 8; allocation, reuse and release as for the
 * scratch buffer below) when the problem has at least 64^3 multiply-adds.  C, bias and
 * rowsum are always used in place, whatever N is and wherever they start (element
 * alignment).  A B given as [K][N] with at most 32 columns (under an output of more than
 * 32 rows) is likewise copied first, in transposed form, so that the product can run on
 * the 128 x 32 tile, and so is an A or B that does not start on a 16-byte boundary.  What
 * is left for a slower, bounds-checked kernel: problems below 64^3 multiply-adds that
 * would need such a copy, and outputs below 16 x 16 with K below 1024.
 * M, N, K must each be below 2^31 and batch*M*N, batch*M*K, batch*K*N below 2^62 (else
 * PGK_ERR_UNSUPPORTED).
 *
 * The library keeps a device scratch buffer per (device, stream), allocated on first
 * use (hipMalloc; PGK_ERR_HIP if that fails), grown when needed, reused afterwards and
 * released by pgk_release_scratch().  It holds the per-tile partial row sums when rowsum
 * is requested and N spans several tile columns, and -- for problems with few output
 * tiles and a long K (a grid that would leave most of the chip idle -- fewer than 192
 * tiles of the shape in use, 384 for the skinny tiles -- and K long enough for at least
 * two slices; or fewer than 192 large tiles and K of at least 512 K tiles; pgk_gemm_plan
 * tells) -- the partial products of an automatic K split, computed exactly as by
 * pgk_gemm_splitk with splits = 0 (at most 256 MiB; larger cases are not split).  Which
 * route a problem takes depends on its shape only, so results stay bit-reproducible.
 */
int pgk_gemm_fused(const void* A, const void* B, const float* bias, void* C, float* rowsum,
                   int64_t M, int64_t N, int64_t K, int64_t batch,
                   int act, int dtype, void* stream);

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
 * workspace: device buffer of at least pgk_splitk_workspace_bytes(...) bytes,
 * 16-byte aligned, owned by the caller, contents destroyed.  Too small or NULL
 * gives PGK_ERR_WORKSPACE.
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
 * and rowsum, ownership, the scratch buffer, the split rule, the workspace size
 * (pgk_splitk_workspace_bytes does not depend on the layout of B) and the errors are as
 * for pgk_gemm_fused / pgk_gemm_splitk.  The matrix-core kernels read Bt in place -- no
 * transposed copy is made -- when its rows start on 4-byte boundaries (float32, or an even
 * K), whatever N is; otherwise A and Bt are copied with K padded, as described there.
 */
int pgk_gemm_fused_bt(const void* A, const void* Bt, const float* bias, void* C, float* rowsum,
                      int64_t M, int64_t N, int64_t K, int64_t batch,
                      int act, int dtype, void* stream);
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

/* Bytes of workspace pgk_gemm_splitk needs for this problem (splits = 0: the
 * automatic choice).  Pure host arithmetic; returns 0 for invalid arguments. */
size_t pgk_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch,
                                  int dtype, int splits);

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
 * second small kernel combines them; the segment results live in the same per
 * (device, stream) scratch buffer as the row-sum partials (hipMalloc on first use).
 * The result does not depend on how the work was split and is bit-reproducible.
 */
int pgk_reduce_max(const void* X, void* out, int32_t* idx,
                   int64_t outer, int64_t red, int64_t inner, int dtype, void* stream);

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
 * pgk_probe_mfma / pgk_probe_stream_read -- measurement aids, not operators: what the chip
 * sustains under its power limit, to read a kernel's numbers against (the paper's Section 3.2
 * lists matrix-unit activity and memory throughput among a performance engineer's evidence).
 *
 * pgk_probe_mfma launches 512 workgroups (two per CU, two waves per SIMD) in which every wave
 * issues iters * 32 matrix instructions of `dtype` on register operands -- all zero
 * (random_operands = 0: nothing toggles, the clock stays high) or random finite values
 * (random_operands = 1: what a real GEMM's operands do to the clock).  *flops_out (host
 * pointer, may be NULL) receives the floating-point operations of one launch.
 * pgk_probe_stream_read reads `bytes` (a multiple of 16, 16-byte aligned device memory at
 * `src`) once with 16-byte loads.  `sink` is one float of device memory for both; it is not
 * written in practice.  Time the calls with events on `stream`.  iters in [1, 2^20].
 */
int pgk_probe_mfma(int dtype, int random_operands, int iters, float* sink, double* flops_out, void* stream);
int pgk_probe_stream_read(const void* src, size_t bytes, float* sink, void* stream);

/* Frees the row-sum scratch buffers of the current process (synchronises the
 * devices that own them).  Optional; safe to call when none exist. */
int pgk_release_scratch(void);

/* Human-readable name of a status code; never NULL.  Host pointer, static storage. */
const char* pgk_status_string(int status);

/* Library version as major*10000 + minor*100 + patch. */
int pgk_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PGK_H */
