/*
 * CPU oracle for the fused GEMM + epilogue operator.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the checker the GPU library is compared against.  It is plain C,
 * evaluates the textbook definition in double precision, and shares no code,
 * header, table or constant with the HIP kernels.  Only the tests, the smoke
 * check and the CPU-baseline leg of the benchmark may call it; the product
 * path never does.
 *
 * What it follows.  PRAGMA (arXiv 2511.06345) is a paper about an agent loop
 * that rewrites operator kernels; Section 1 (Introduction) and Section 4.1
 * (Datasets) name the operator families (matrix multiplication, element-wise /
 * activation, reduction) and give no formula for them.  The operator checked
 * here is therefore the plain mathematical definition:
 *
 *     x[b,i,j]    = bias[j] + sum_{k=0}^{K-1} A[b,i,k] * B[b,k,j]
 *     y[b,i,j]    = act(x[b,i,j])
 *     C[b,i,j]    = y[b,i,j]
 *     rowsum[b,i] = sum_{j=0}^{N-1} y[b,i,j]
 *
 * with act one of identity, ReLU, tanh-form GELU and SiLU (standard published
 * forms, written out below).  Everything is accumulated and returned in
 * double; nothing is rounded to the storage type, so C and rowsum are the
 * real-number result up to double rounding.
 *
 * Pins (see tests): hand-computed 2x2 case, identity / permutation operands,
 * all-ones closed form, integer-exact agreement with int64 arithmetic,
 * linearity and transpose invariants, the mat-vec closed form of rowsum, a
 * float64 library matmul on random shapes, and tabulated activation values.
 * No function in this file is "parity unpinned".
 *
 * Second operator: maximum over one dimension (the paper's GPU case study,
 * Section 4.4 "Max reduction over a dimension"; the paper gives no formula or
 * shape).  oracle_reduce_max below is the definition written out as one scan
 * per output element.  Pins (see tests): agreement with numpy's max / argmax,
 * hand cases, "attained, not exceeded, nothing equal before it", invariance
 * of the value under permutation of the reduced axis, reduced length 1, ties
 * between +0 and -0, NaN and infinity cases.
 *
 * Third operator: one-dimensional convolution (the paper's second case study,
 * Section 4.4 "Conv Standard 1D"; again no formula or shape is given).
 * oracle_conv1d is the definition as used by deep-learning frameworks
 * (cross-correlation with zero padding, stride and dilation), four nested loops
 * in double.  Pins (see tests): numpy's correlate on every channel pair, a
 * kernel of width one against the matrix product, unit-impulse kernels (pure
 * shifts), the all-ones closed form that counts the taps inside the input,
 * linearity, shift equivariance, integer-exact agreement with int64.
 *
 * Loop order is (b, i, k, j) with one row of N double accumulators, so the
 * inner loop is stride-1 in B; rows are independent and are shared among
 * OpenMP threads.  No blocking, no fusion beyond the definition.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_RELU = 1, ORACLE_ACT_GELU_TANH = 2, ORACLE_ACT_SILU = 3 };
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* bfloat16 is the upper 16 bits of an IEEE binary32; widening is exact. */
static double bf16_to_double(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Activation functions in double.
 *   ReLU(x)      = max(x, 0), with ReLU(-0) = +0
 *   GELU_tanh(x) = 0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) ))
 *   SiLU(x)      = x / (1 + exp(-x))
 */
double oracle_act(double x, int act)
{
    switch (act) {
    case ORACLE_ACT_NONE:
        return x;
    case ORACLE_ACT_RELU:
        return x > 0.0 ? x : 0.0;
    case ORACLE_ACT_GELU_TANH: {
        const double c = 0.7978845608028654; /* sqrt(2/pi) */
        double u = c * (x + 0.044715 * x * x * x);
        return 0.5 * x * (1.0 + tanh(u));
    }
    case ORACLE_ACT_SILU:
        return x / (1.0 + exp(-x));
    default:
        return NAN;
    }
}

static double load_elem(const void *p, int dtype, int64_t idx)
{
    if (dtype == ORACLE_BF16)
        return bf16_to_double(((const uint16_t *)p)[idx]);
    return (double)((const float *)p)[idx];
}

/*
 * oracle_gemm_fused
 *   A      [batch][M][K]  row-major, float32 (dtype 0) or bfloat16 bit patterns (dtype 1)
 *   B      [batch][K][N]  row-major, same type as A
 *   bias   [N] float32, or NULL meaning zero
 *   rows   list of nrows row indices in [0,M) to evaluate, or NULL meaning all
 *          M rows in order (then nrows is ignored)
 *   C_out  [batch][R][N] double, R = nrows (or M); may be NULL
 *   rs_out [batch][R]    double; may be NULL
 * Returns 0, or -1 on an invalid argument.
 */
int oracle_gemm_fused(const void *A, const void *B, const float *bias,
                      int64_t M, int64_t N, int64_t K, int64_t batch,
                      int act, int dtype,
                      const int64_t *rows, int64_t nrows,
                      double *C_out, double *rs_out)
{
    if (!A || !B || M <= 0 || N <= 0 || K <= 0 || batch <= 0) return -1;
    if (act < 0 || act > 3 || (dtype != ORACLE_F32 && dtype != ORACLE_BF16)) return -1;
    const int64_t R = rows ? nrows : M;
    if (R <= 0) return -1;
    if (rows)
        for (int64_t r = 0; r < R; ++r)
            if (rows[r] < 0 || rows[r] >= M) return -1;

    const int64_t total = batch * R;
    int failed = 0;
#pragma omp parallel
    {
        double *acc = (double *)malloc((size_t)N * sizeof(double));
        if (!acc) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t t = 0; t < total; ++t) {
            if (!acc) continue;
            const int64_t b = t / R;
            const int64_t r = t % R;
            const int64_t i = rows ? rows[r] : r;
            for (int64_t j = 0; j < N; ++j) acc[j] = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const double a = load_elem(A, dtype, (b * M + i) * K + k);
                const int64_t brow = (b * K + k) * N;
                if (dtype == ORACLE_BF16) {
                    const uint16_t *Bp = (const uint16_t *)B + brow;
                    for (int64_t j = 0; j < N; ++j) acc[j] += a * bf16_to_double(Bp[j]);
                } else {
                    const float *Bp = (const float *)B + brow;
                    for (int64_t j = 0; j < N; ++j) acc[j] += a * (double)Bp[j];
                }
            }
            double s = 0.0;
            for (int64_t j = 0; j < N; ++j) {
                const double x = acc[j] + (bias ? (double)bias[j] : 0.0);
                const double y = oracle_act(x, act);
                if (C_out) C_out[(b * R + r) * N + j] = y;
                s += y;
            }
            if (rs_out) rs_out[b * R + r] = s;
        }
        free(acc);
    }
    return failed ? -1 : 0;
}

/*
 * Maximum over the middle dimension of X viewed as [outer][red][inner]
 * (row-major, contiguous), which covers a reduction over any one dimension of a
 * contiguous tensor:
 *
 *     out[o][i] = max_{r} X[o][r][i]
 *     idx[o][i] = the smallest r with X[o][r][i] == out[o][i]
 *
 * under IEEE comparison (+0 and -0 compare equal, so the earlier one is
 * returned).  If the slice holds a NaN the result is that NaN and idx the
 * position of the first NaN.  Values are returned widened to float (exact for
 * both storage types), idx may be NULL.  Returns 0, or -1 for bad arguments.
 */
int oracle_reduce_max(const void *X, int dtype, int64_t outer, int64_t red, int64_t inner,
                      float *out, int32_t *idx)
{
    if (!X || !out || outer <= 0 || red <= 0 || inner <= 0 || red > 2147483647LL) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t i = 0; i < inner; ++i) {
            const int64_t base = o * red * inner + i;
            float best = (float)load_elem(X, dtype, base);
            int64_t at = 0;
            for (int64_t r = 1; r < red && best == best; ++r) {      /* a NaN ends the scan */
                const float x = (float)load_elem(X, dtype, base + r * inner);
                if (x != x || x > best) { best = x; at = r; }
            }
            out[o * inner + i] = best;
            if (idx) idx[o * inner + i] = (int32_t)at;
        }
    }
    return 0;
}

/*
 * One-dimensional convolution with bias and activation:
 *
 *     y[b][co][l] = act( bias[co] + sum_{ci} sum_{k} w[co][ci][k] * x[b][ci][l*stride + k*dilation - pad] )
 *
 * where x outside [0, L) counts as zero, and
 *     Lout = floor((L + 2 pad - dilation (Kw - 1) - 1) / stride) + 1.
 *   x [B][Cin][L], w [Cout][Cin][Kw] row-major, float32 or bfloat16 bits (dtype);
 *   bias [Cout] float32 or NULL; y_out [B][Cout][Lout] double, nothing rounded.
 * Returns Lout, or -1 for bad arguments (including Lout <= 0).
 */
int64_t oracle_conv1d(const void *x, const void *w, const float *bias, int dtype,
                      int64_t B, int64_t Cin, int64_t L, int64_t Cout, int64_t Kw,
                      int64_t stride, int64_t pad, int64_t dilation, int act, double *y_out)
{
    if (!x || !w || !y_out || B <= 0 || Cin <= 0 || L <= 0 || Cout <= 0 || Kw <= 0) return -1;
    if (stride <= 0 || pad < 0 || dilation <= 0) return -1;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -1;
    if (act < ORACLE_ACT_NONE || act > ORACLE_ACT_SILU) return -1;
    const int64_t span = L + 2 * pad - dilation * (Kw - 1) - 1;
    if (span < 0) return -1;
    const int64_t Lout = span / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t co = 0; co < Cout; ++co) {
            for (int64_t l = 0; l < Lout; ++l) {
                double acc = bias ? (double)bias[co] : 0.0;
                for (int64_t ci = 0; ci < Cin; ++ci) {
                    for (int64_t k = 0; k < Kw; ++k) {
                        const int64_t pos = l * stride + k * dilation - pad;
                        if (pos < 0 || pos >= L) continue;
                        acc += load_elem(w, dtype, (co * Cin + ci) * Kw + k) *
                               load_elem(x, dtype, (b * Cin + ci) * L + pos);
                    }
                }
                y_out[(b * Cout + co) * Lout + l] = oracle_act(acc, act);
            }
        }
    }
    return Lout;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
