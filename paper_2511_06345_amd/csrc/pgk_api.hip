// C-ABI layer of libpgk: argument validation (host only, before any HIP call),
// choice of kernel path and launch geometry, and the layout of the caller's workspace.
// The library allocates no device memory and keeps no state between calls.
// The contract of every entry point is documented in include/pgk.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>

#include "../../include/pgk.h"
#include "pgk_kernels.h"

// The fixed workspace of pgk_gemm_fused_static (device memory; see static_scratch_of_current_device).
static __device__ __align__(256) unsigned char scratch[(size_t)4 << 20];

namespace {

using pgk::GemmArgs;

constexpr int64_t kMaxDim = 0x7fffffffLL;
constexpr int kNumCUs = 256;          // MI355X
// Shortest slice of an automatic split, in K tiles: below that the second pass and launch cost
// more than the shorter loop saves.  16; for bf16, whose K tile takes half as long as an fp32
// one, 32 once the small-tile grid has 96 workgroups (with slices of 16: 1024 x 2048 x 2048 27 us
// in two slices, 20 us in one, 1536 x 1536 x 4096 45 us in four, 41 us in two; but 768 x 768 x 3072,
// 36 tiles, 22 us in three and 32 us in one; fp32 512 x 512 x 1024 18 us in two, 22 us in one).
int min_steps_per_slice(int dtype, long double small_tiles) { return dtype == PGK_DTYPE_BF16 && small_tiles >= 96 ? 32 : 16; }
constexpr size_t kAutoSplitMaxWorkspace = (size_t)256 << 20;   // workspace pgk_gemm_fused may ask for an automatic split
constexpr int kMaxAutoSplits = 32;
constexpr int64_t kLongKSteps = 512;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate_common(const void* A, const void* B, const void* C, int64_t M, int64_t N, int64_t K,
                    int64_t batch, int act, int dtype)
{
    if (!A || !B || !C) return PGK_ERR_INVALID_ARG;
    if (M <= 0 || N <= 0 || K <= 0 || batch <= 0) return PGK_ERR_INVALID_ARG;
    if (act < PGK_ACT_NONE || act > PGK_ACT_SILU) return PGK_ERR_INVALID_ARG;
    if (dtype != PGK_DTYPE_F32 && dtype != PGK_DTYPE_BF16) return PGK_ERR_INVALID_ARG;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim || batch > kMaxDim) return PGK_ERR_UNSUPPORTED;
    const long double lim = 4.6e18L;  // 2^62
    if ((long double)batch * M * N >= lim || (long double)batch * M * K >= lim ||
        (long double)batch * K * N >= lim)
        return PGK_ERR_UNSUPPORTED;
    return PGK_OK;
}

int kstep_of(int dtype) { return pgk::mfma_tile_shape(dtype, false).bk; }

// Split geometry shared by the workspace query and the launch: slice length L
// and the number of non-empty slices.
struct SplitPlan { int splits; int k_slice; };

size_t round_up256(size_t v) { return (v + 255) / 256 * 256; }
int64_t chunk_elems(int dtype) { return dtype == PGK_DTYPE_BF16 ? 8 : 4; }
int64_t round_up64(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

// What the matrix-core kernels take as it is: operand rows that start on 4-byte boundaries (K
// elements for A and a transposed B; the row length ldb of a plain B, which is N unless the
// caller has padded it).  M, N and K need not be tile multiples, and the output rows may have any
// length.  An
// output below 16 x 16 is left to the bounds-checked kernel, which wastes less, unless K is
// long (then the matrix-core route splits the K range over the chip).
bool mfma_shape_ok(int64_t M, int64_t N, int64_t K, int dtype, bool b_trans = false, int64_t ldb = 0)
{
    const pgk::TileShape t = pgk::mfma_tile_shape(dtype, false);
    const int64_t es = dtype == PGK_DTYPE_BF16 ? 2 : 4;
    if (!ldb) ldb = b_trans ? K : N;
    if ((K * es) % 4 || (ldb * es) % 4) return false;
    if (M < 16 && N < 16 && K < 1024) return false;
    // per-lane 32-bit byte offsets inside one tile
    if ((int64_t)t.bm * K * es >= (1LL << 32)) return false;
    if ((b_trans ? (int64_t)t.bn * K : (int64_t)t.bk * ldb) * es >= (1LL << 32)) return false;
    return true;
}

// Operand rows that would start off 4-byte boundaries (bf16: an odd K, or an odd N for a plain
// B): the operands are first copied into buffers with rows padded with zeros to whole 16-byte
// chunks.  Worth it from about 64^3 multiply-adds on.
bool needs_packing(int64_t N, int64_t K, int dtype, bool b_trans)
{
    const int64_t es = dtype == PGK_DTYPE_BF16 ? 2 : 4;
    return (K * es) % 4 != 0 || (!b_trans && (N * es) % 4 != 0);
}

// Outputs with at most 32 columns or rows: the skinny tiles (narrow 128 x 32, flat 32 x 128), on
// which such a product stays bound by the stream of its large operand instead of by matrix work
// on padding (bf16 16384 x 16 x 16384: 137 us on 128 x 128 tiles).  The narrow tile exists for a
// transposed B only; a plain B of so few columns is small and is transposed first (see route_for).
// -1: not skinny.
int skinny_tile_kind(int64_t M, int64_t N)
{
    if (M <= 32 && N > 32) return pgk::TILE_FLAT;
    if (N <= 32 && M > 32) return pgk::TILE_NARROW;
    if (M <= 32 && N <= 32) return pgk::TILE_FLAT;
    return -1;
}

// The dimensions the kernels see for a problem that is packed first: K and the row length of B,
// rounded up to whole chunks where they are odd.  pack = false: the problem is taken as it is (aligned already, or
// too small or too large for this to pay).
// transpose_b: a plain B of at most 32 columns under more than 32 rows of output is copied in
// transposed form, [N][k], for the narrow tile; the kernels then see a transposed B (b_trans).
struct PackDims { bool pack; int64_t k, ldb; bool transpose_b; bool b_trans; };

// misaligned: A or B does not start on a 16-byte boundary; the copies do (pack_operands copies
// whichever operand needs it), and their rows are whole chunks.
PackDims pack_dims(int64_t M, int64_t N, int64_t K, int dtype, bool b_trans, bool misaligned = false)
{
    const PackDims as_is{false, K, 0, false, b_trans};
    const bool transpose_b = !b_trans && skinny_tile_kind(M, N) == pgk::TILE_NARROW;
    if (!transpose_b && !misaligned && !needs_packing(N, K, dtype, b_trans)) return as_is;
    if ((long double)M * N * K < 262144.0L) return as_is;
    const int64_t epc = chunk_elems(dtype), es = dtype == PGK_DTYPE_BF16 ? 2 : 4;
    PackDims d{true, ((K * es) % 4 || misaligned) ? round_up64(K, epc) : K, 0, transpose_b, b_trans || transpose_b};
    // (a plain B is copied in every such case; so is a B that is transposed, with rows of whole chunks)
    d.ldb = transpose_b ? round_up64(d.k, epc) : d.b_trans ? d.k : round_up64(N, epc);
    if (d.k > kMaxDim || d.ldb > kMaxDim) return as_is;
    if (!mfma_shape_ok(M, N, d.k, dtype, d.b_trans, d.ldb)) return as_is;
    return d;
}

// the plan queries, which do not know the layout of B: does this problem end up on the matrix
// cores, one way or the other, with either layout
bool mfma_route(int64_t M, int64_t N, int64_t K, int dtype)
{
    return mfma_shape_ok(M, N, K, dtype) || pack_dims(M, N, K, dtype, false).pack ||
           mfma_shape_ok(M, N, K, dtype, true) || pack_dims(M, N, K, dtype, true).pack;
}

// A large tile mostly outside the matrix (skinny M or N): the small tile wastes less matrix work
// and fewer operand loads.  bf16: three quarters empty (between a quarter and a half full the
// half tiles take over; 128 x 65536 x 1024 took 35 us with the large tile, 28 us with either the
// small or the half one).  fp32, which has no half tiles: half empty -- 64 x 65536 x 1024 took
// 146 us with the large tile and 78 us with the small one, 96 x 65536 x 1024 133 and 146 us.
bool large_tile_mostly_empty(int64_t M, int64_t N, int dtype)
{
    const pgk::TileShape big = pgk::mfma_tile_shape(dtype, false);
    const int64_t f = dtype == PGK_DTYPE_BF16 ? 4 : 2;
    return f * M <= big.bm || f * N <= big.bn;
}

// How long a grid of one tile shape takes, in rounds: the chip runs per_cu workgroups per CU
// side by side, a full round of them takes fixed + per_k * K / 1024 (microseconds on the
// measured part; only ratios between shapes are used), and a last, partly filled round with j
// workgroups on its busiest CU takes the share tail[j - 1] of a full one.  Fitted to GEMMs of
// 2560^2 ... 8192^2 outputs with K = 1024 ... 4096 (e.g. bf16 4096^2 x 4096: 256 large tiles 104 us,
// 1024 small ones 122 us, 512 half tiles 114 us; fp32: 1024 large 913 us, 4096 small 965 us).
struct TileCost { int per_cu; double fixed, per_k; double tail[4]; };

TileCost tile_cost(int dtype, int kind)
{
    if (dtype == PGK_DTYPE_BF16) {
        switch (kind) {
        case pgk::TILE_SMALL: return {2, 2.9, 14.3, {0.47, 1.0, 1.0, 1.0}};
        case pgk::TILE_TALL: return {1, 5.8, 12.8, {0.65, 1.0, 1.0, 1.0}};
        case pgk::TILE_WIDE: return {1, 5.7, 13.2, {0.65, 1.0, 1.0, 1.0}};
        default: return {1, 10.0, 22.5, {0.7, 1.0, 1.0, 1.0}};
        }
    }
    if (kind == pgk::TILE_SMALL) return {4, 1.5, 59.9, {0.3, 0.6, 0.75, 1.0}};
    return {1, 3.0, 56.2, {1.0, 1.0, 1.0, 1.0}};
}

double estimated_rounds_time(int64_t M, int64_t N, int64_t K, int dtype, int64_t units, int kind)
{
    const pgk::TileShape t = pgk::mfma_tile_shape(dtype, kind);
    const TileCost c = tile_cost(dtype, kind);
    const double wgs = (double)((M + t.bm - 1) / t.bm) * (double)((N + t.bn - 1) / t.bn) * (double)units;
    const double slots = (double)kNumCUs * c.per_cu;
    const double full = std::floor(wgs / slots), rest = wgs - full * slots;
    const int j = (int)std::ceil(rest / kNumCUs);
    return (c.fixed + c.per_k * (double)K / 1024.0) * (full + (j > 0 ? c.tail[j - 1] : 0.0));
}

// Automatic choice (splits == 0): slices of at least min_steps_per_slice K steps (shorter ones
// are all prologue and epilogue), at most kMaxAutoSplits of them, and the smallest count that
// gives 2 x 256 workgroups.  The tile the count is made with: a skinny one for skinny outputs,
// else the large one if it can reach 1.5 x 256 workgroups within those limits and is not mostly
// empty, else the small one.
struct AutoPlan { int splits; int kind; };

AutoPlan auto_split(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype)
{
    const int ks = kstep_of(dtype);
    const int64_t ksteps = (K + ks - 1) / ks;
    auto tiles_of = [&](int kind) {
        const pgk::TileShape t = pgk::mfma_tile_shape(dtype, kind);
        return (long double)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn) * batch;
    };
    // (outputs of at most 64 rows or columns are bound by the stream of their large operand, which
    // more workgroups pull harder on: 16 K tiles per slice for them in any case)
    int64_t s_max = ksteps / ((M <= 64 || N <= 64) ? 16 : min_steps_per_slice(dtype, tiles_of(pgk::TILE_SMALL)));
    if (s_max < 1) s_max = 1;
    if (s_max > kMaxAutoSplits) s_max = kMaxAutoSplits;
    int kind = skinny_tile_kind(M, N);
    if (kind < 0)
        kind = (large_tile_mostly_empty(M, N, dtype) || tiles_of(pgk::TILE_LARGE) * s_max < 1.5L * kNumCUs) ? pgk::TILE_SMALL
                                                                                                          : pgk::TILE_LARGE;
    const long double tiles = tiles_of(kind);
    // (enough slices for two workgroups per CU; four of the fp32 small tile and one of the bf16
    // large tile, which is how many of those fit a CU: a second round of half-length slices does
    // the same matrix work and doubles the partial products -- bf16 1024 x 2048 x 16384 took 100 us
    // in 16 slices and 78 us in 8)
    const long double target = (dtype == PGK_DTYPE_F32 && kind == pgk::TILE_SMALL   ? 4.0L
                                : dtype == PGK_DTYPE_BF16 && kind == pgk::TILE_LARGE ? 1.0L
                                                                                      : 2.0L) * kNumCUs;
    auto slices_for = [&](long double n_tiles, long double goal) {
        int64_t n = 1;
        while (n < s_max && n_tiles * n < 0.95L * goal) ++n;      // (250 tiles: two slices, not three)
        return n;
    };
    int64_t s = slices_for(tiles, target);
    // Large against small tile once more, now with their slice counts, by the round model (plus
    // what the partial products cost: written and read once, at about 4 TB/s, and a launch): the
    // rule above takes the large tile whenever it can fill the chip, also when its grid then ends
    // in a poorly filled round or needs many more slices (fp32 1536 x 1536 x 8192: 144 large tiles
    // x 4 slices = 2.25 rounds, 357 us; 576 small tiles x 2 slices 313 us).  Slices of 1024 K
    // values and more only: that is what the model was fitted to.
    if (kind == pgk::TILE_LARGE || kind == pgk::TILE_SMALL) {
        auto estimate = [&](int knd, int64_t n) {
            const double second_pass = 2.0 * (double)n * (double)M * (double)N * (double)batch * 4.0 / 4.0e6 + 5.0;
            return estimated_rounds_time(M, N, (K + n - 1) / n, dtype, batch * n, knd) + (n > 1 ? second_pass : 0.0);
        };
        const int other = kind == pgk::TILE_LARGE ? pgk::TILE_SMALL : pgk::TILE_LARGE;
        const long double other_target = (dtype == PGK_DTYPE_F32 && other == pgk::TILE_SMALL   ? 4.0L
                                          : dtype == PGK_DTYPE_BF16 && other == pgk::TILE_LARGE ? 1.0L
                                                                                                 : 2.0L) * kNumCUs;
        const int64_t s_other = slices_for(tiles_of(other), other_target);
        const bool other_allowed = other == pgk::TILE_SMALL || !large_tile_mostly_empty(M, N, dtype);
        if (other_allowed && K / s >= 1024 && K / s_other >= 1024 && estimate(other, s_other) < 0.94 * estimate(kind, s)) {
            kind = other;
            s = s_other;
        }
    }
    return {(int)s, kind};
}

SplitPlan plan_splits(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int splits)
{
    const int ks = kstep_of(dtype);
    const int64_t ksteps = (K + ks - 1) / ks;
    int64_t s = splits;
    if (s == 0) {
        if (mfma_route(M, N, K, dtype)) {
            s = auto_split(M, N, K, batch, dtype).splits;
        } else {
            const pgk::TileShape t = pgk::guarded_tile_shape();
            const long double tiles = (long double)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn) * batch;
            s = 1;
            while (s < kMaxAutoSplits && s < ksteps && tiles * s < 2.0L * kNumCUs) ++s;
        }
    }
    if (s > ksteps) s = ksteps;
    const int64_t per = (ksteps + s - 1) / s;     // K steps per slice
    const int64_t L = per * ks;
    const int64_t eff = (K + L - 1) / L;          // drop trailing empty slices
    return {(int)eff, (int)L};
}

int group_m_for(int tiles_m, int tiles_n)
{
    // 32 workgroups of an XCD run together; keep their tiles near-square.
    int g = tiles_n >= 8 ? 4 : 8;
    if (g > tiles_m) g = tiles_m;
    return g;
}

struct Path { bool mfma; int kind; pgk::TileShape tile; };

// Half of a large tile (tall: half as wide; wide: half as high) when that takes away at least
// a third of the padded area the large tiles would compute -- the last tile column or row at
// most half full and few of them -- and still gives a grid that fills the chip.  (With less
// padding to save the large tile's better main loop wins: a half tile moves three quarters of
// the operand bytes per K tile for half the matrix work.)
int half_tile_kind(int64_t M, int64_t N, int dtype, int64_t units, bool b_trans)
{
    const pgk::TileShape big = pgk::mfma_tile_shape(dtype, pgk::TILE_LARGE);
    const long double area_large = (long double)((M + big.bm - 1) / big.bm * big.bm) * ((N + big.bn - 1) / big.bn * big.bn);
    for (int kind : {pgk::TILE_TALL, pgk::TILE_WIDE}) {
        if (!pgk::mfma_has_tile(dtype, kind, b_trans)) continue;
        const pgk::TileShape t = pgk::mfma_tile_shape(dtype, kind);
        const int64_t tm = (M + t.bm - 1) / t.bm, tn = (N + t.bn - 1) / t.bn;
        const long double area = (long double)(tm * t.bm) * (tn * t.bn);
        if (3 * area <= 2 * area_large && (long double)tm * tn * units >= 0.75L * kNumCUs) return kind;
    }
    return -1;
}

// The tile shape for an output of M x N with `units` workgroups per tile position (batch entries
// x K splits): the small tile when three quarters of a large tile would be empty, else a half
// tile when that saves a third of the padding, else the small tile when the large-tile grid would
// leave a quarter of the CUs idle or K is at most two bf16 K tiles, else the large tile -- unless its grid ends in a poorly
// filled round and the round model above gives another shape at least 6 % less time (K below
// 1024: the model is not consulted).
// Latency-bound fp32 problems: so few 64 x 64 tiles that most of the chip would idle behind one
// chain of K/2 dependent matrix instructions per wave, and a K too short for a two-pass split.
// They run on 32 x 32 tiles whose four waves split the K range (256 x 256 x 256: 16 workgroups
// with chains of 128 instructions become 64 workgroups with chains of 32).
bool tiny_problem(int64_t M, int64_t N, int64_t K, int dtype, int64_t units, bool b_trans, int64_t ldb)
{
    if (dtype != PGK_DTYPE_F32 || b_trans || K < 64 || K % 4 || N % 4 || (ldb ? ldb : N) % 4) return false;
    if (M <= 32 || N <= 32) return false;                       // (the skinny tiles' business)
    const long double tiles64 = (long double)((M + 63) / 64) * ((N + 63) / 64) * units;
    const int64_t ksteps = (K + 31) / 32;
    return tiles64 <= 64.0L && ksteps < 2 * 16;                 // (from 2 x 16 K tiles on, the K range is split in two passes)
}

int auto_tile_kind(int64_t M, int64_t N, int64_t K, int dtype, int64_t units, bool b_trans, int64_t ldb = 0)
{
    // (K = 0: a convolution, which keeps to the shapes its operand views were written for)
    if (const int skinny = skinny_tile_kind(M, N); K > 0 && skinny >= 0 && pgk::mfma_has_tile(dtype, skinny, b_trans)) return skinny;
    if (K > 0 && tiny_problem(M, N, K, dtype, units, b_trans, ldb)) return pgk::TILE_TINY;
    if (large_tile_mostly_empty(M, N, dtype)) return pgk::TILE_SMALL;
    if (const int half = half_tile_kind(M, N, dtype, units, b_trans); half >= 0) return half;
    // One or two bf16 K tiles: there is no main loop for the large tile to be good at, and two small
    // workgroups per CU overlap one's copies and stores with the other's (8192 x 8192 x 64 46 -> 39 us,
    // 96 x [1024 x 1024 x 64] 58 -> 52 us).  Not with output rows of 32 KiB and more, where the 256-byte
    // pieces of a small tile's rows lie too far apart for the memory (16384 x 16384 x 128: 158 against 171 us).
    if (dtype == PGK_DTYPE_BF16 && K > 0 && K <= 128 && N < 16384) return pgk::TILE_SMALL;
    const pgk::TileShape big = pgk::mfma_tile_shape(dtype, false);
    const long double wgs = (long double)((M + big.bm - 1) / big.bm) * ((N + big.bn - 1) / big.bn) * units;
    if (dtype == PGK_DTYPE_BF16) {
        // One large tile fits a CU, two small ones, one half tile.  Up to half the CUs' worth of
        // large tiles the half and small tiles still run in a single round and win (2560 x 3072 x
        // 4096, 120 large tiles: 75 us large, 62 small, 55 tall); one large tile more and they
        // need a second round while the large tiles do not (2816 x 3072 x 4096, 132: 78 us large,
        // 86 small, 100 tall; the same up to 196).  With at least 192 of them the tall tile is
        // the better single round from 16 K tiles on (5-12 % ahead of the small one).
        if (wgs <= 0.5L * kNumCUs)
            return (K >= 1024 && 2 * wgs >= 0.75L * kNumCUs && pgk::mfma_has_tile(dtype, pgk::TILE_TALL, b_trans)) ? pgk::TILE_TALL
                                                                                                                : pgk::TILE_SMALL;
    } else if (wgs < 0.75L * kNumCUs) {
        return pgk::TILE_SMALL;
    }
    int best = pgk::TILE_LARGE;
    if (K >= 1024 && wgs > kNumCUs) {      // (the fit does not hold for short K, where the epilogues weigh more)
        double best_time = 0.94 * estimated_rounds_time(M, N, K, dtype, units, pgk::TILE_LARGE);
        for (int kind : {pgk::TILE_SMALL, pgk::TILE_TALL, pgk::TILE_WIDE}) {
            if (!pgk::mfma_has_tile(dtype, kind, b_trans)) continue;
            const double t = estimated_rounds_time(M, N, K, dtype, units, kind);
            if (t < best_time) { best_time = t; best = kind; }
        }
    }
    return best;
}

// kind_forced: -1 = auto_tile_kind, else the caller (an automatic split plan, a convolution plan) decides.
// `aligned`: A, B and the split-K partial products start on 16-byte boundaries (C, the biases and
// the row sums only need the alignment of their elements: a row of C may start anywhere, so its
// 16-byte stores are element-aligned ones in any case).
Path choose_path(bool aligned, int64_t M, int64_t N, int64_t K, int dtype, int64_t units, int kind_forced = -1,
                 bool b_trans = false, int64_t ldb = 0)
{
    const bool ok = aligned && mfma_shape_ok(M, N, K, dtype, b_trans, ldb);
    if (!ok) return Path{false, false, pgk::guarded_tile_shape()};
    int kind = kind_forced >= 0 ? kind_forced : auto_tile_kind(M, N, K, dtype, units, b_trans, ldb);
    if (!pgk::mfma_has_tile(dtype, kind, b_trans)) kind = pgk::TILE_SMALL;      // (the narrow tile with a plain B)
    return Path{true, kind, pgk::mfma_tile_shape(dtype, kind)};
}

// rows of B (of Bt) `ldb` elements apart instead of N (of K)
void set_ldb(GemmArgs& a, int64_t ldb)
{
    a.ldb = (int)ldb;
    a.b_batch_stride = (long long)(a.b_trans ? a.N : a.K) * ldb;
}

// call when the views are final: the rows of a plain B that are not whole chunks
void mark_ragged_rows(GemmArgs& a, int dtype)
{
    a.b_tail_bounded = (!a.b_trans && a.ldb % chunk_elems(dtype) != 0) ? 1 : 0;
}

// One tile column (or, with a transposed B, one tile row): the workgroups stream disjoint rows of
// the large operand, K along the rows, and share only the small one.  Their K loops then start
// at different tiles, so that power-of-two row strides do not send every workgroup to the same
// memory channels at once.  With several batch entries the starting tile goes by entry: the
// workgroups of one entry share its small operand and walk K together (rotated against each
// other they fetched it several times: 32 x [2048 x 128 x 2048] bf16 47 -> 53 us).  Not when a single
// entry's shared operand is too large to stay in L2 (walking K in step, they fetch each of its
// tiles once), not with several tile columns and rows (they
// share panels of both operands), and not for a tile row over a plain B, which reads whole rows
// of B side by side with its neighbours -- the pattern the memory likes best (16 x 16384 x 16384
// fp32: 183 us, rotated 214 us).  Whole K tiles only: a partial tile has to come last.
void mark_k_rotation(GemmArgs& a, int dtype, const pgk::TileShape& t)
{
    const long double es = dtype == PGK_DTYPE_BF16 ? 2 : 4, small = 2.0e6L;
    // (with several batch entries the rotation goes by entry and the tiles of one entry stay in
    // step, so the size of what they share does not matter)
    const bool streams_a = a.tiles_n == 1 && a.tiles_m > 1 && (a.batch > 1 || (long double)a.K * a.N * es <= small);
    const bool streams_bt = a.tiles_m == 1 && a.tiles_n > 1 && a.b_trans && (a.batch > 1 || (long double)a.K * a.M * es <= small);
    a.k_rotate = ((streams_a || streams_bt) && a.K % t.bk == 0 && a.k_slice % t.bk == 0 && !a.b_tail_bounded) ? 1 : 0;
}

// The two passes of the split-K path.  `workspace`: batch * plan.splits * M * N floats;
// `part`: batch * nseg * M floats when rowsum != nullptr and the second pass uses nseg > 1
// column segments (nseg from splitk_reduce_segments), else unused.  A, B and the workspace
// start on 16-byte boundaries.
int run_split_passes(const void* A, const void* B, const float* bias, void* C, float* rowsum, int64_t M, int64_t N,
                     int64_t K, int64_t batch, int act, int dtype, const SplitPlan& plan, int small_tile,
                     float* workspace, float* part, hipStream_t st, bool aligned, bool b_trans, int64_t ldb = 0)
{
    Path path = choose_path(aligned, M, N, K, dtype, batch * plan.splits, small_tile, b_trans, ldb);
    // (the K-splitting tile of latency-bound problems has no first-pass form: its slices are its waves)
    if (path.mfma && path.kind == pgk::TILE_TINY)
        path = choose_path(aligned, M, N, K, dtype, batch * plan.splits, pgk::TILE_SMALL, b_trans, ldb);
    const int64_t tiles_m = (M + path.tile.bm - 1) / path.tile.bm;
    const int64_t tiles_n = (N + path.tile.bn - 1) / path.tile.bn;
    if ((long double)tiles_m * tiles_n * batch * plan.splits > 2.0e9L) return PGK_ERR_UNSUPPORTED;

    GemmArgs a{};
    a.A = A; a.B = B; a.bias = nullptr; a.C = nullptr; a.rs_part = nullptr;
    a.ws = workspace;
    a.M = (int)M; a.N = (int)N; a.K = (int)K; a.batch = (int)batch;
    pgk::fill_plain_views(a);
    if (b_trans) pgk::set_b_transposed(a);
    if (ldb) set_ldb(a, ldb);
    mark_ragged_rows(a, dtype);
    a.act = PGK_ACT_NONE; a.splits = plan.splits; a.k_slice = plan.k_slice;
    a.tiles_m = (int)tiles_m; a.tiles_n = (int)tiles_n;
    a.group_m = group_m_for(a.tiles_m, a.tiles_n);

    if (path.mfma) mark_k_rotation(a, dtype, path.tile);
    hipError_t e = path.mfma ? pgk::launch_gemm_mfma(a, dtype, path.kind, 1, st) : pgk::launch_gemm_guarded(a, dtype, 1, st);
    if (e != hipSuccess) return PGK_ERR_HIP;
    const int nseg = pgk::splitk_reduce_segments((int)M, (int)N, (int)batch);
    float* rs_part = (rowsum && nseg > 1) ? part : nullptr;
    e = pgk::launch_splitk_reduce(a.ws, bias, C, rowsum, rs_part, nseg, (int)M, (int)N, (int)batch, plan.splits, act, dtype, st);
    if (e != hipSuccess) return PGK_ERR_HIP;
    if (rs_part) e = pgk::launch_rowsum_combine(rs_part, rowsum, (int)M, (int)batch, nseg, st);
    return e == hipSuccess ? PGK_OK : PGK_ERR_HIP;
}

size_t split_part_bytes(int64_t M, int64_t N, int64_t batch, bool rowsum)
{
    const int nseg = pgk::splitk_reduce_segments((int)M, (int)N, (int)batch);
    return (rowsum && nseg > 1) ? (size_t)batch * (size_t)nseg * (size_t)M * sizeof(float) : 0;
}

// What pgk_gemm_fused does with a problem: the kernel and tile of the single-pass route, and
// whether the K range is split instead (then `slices` and the tile that goes with them).
struct FusedPlan {
    Path path;
    bool split;
    SplitPlan slices;
    int split_small_tile;
};

FusedPlan plan_fused(bool aligned, int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, bool b_trans, int64_t ldb = 0)
{
    FusedPlan fp{};
    fp.path = choose_path(aligned, M, N, K, dtype, batch, -1, b_trans, ldb);
    const int64_t tiles_m = (M + fp.path.tile.bm - 1) / fp.path.tile.bm;
    const int64_t tiles_n = (N + fp.path.tile.bn - 1) / fp.path.tile.bn;
    // Few output tiles and a long K (skinny or small outputs): one workgroup per tile would
    // leave most of the chip idle, so the K range is split as in pgk_gemm_splitk, with the
    // partial products in the caller's workspace.  The choice depends on the shape only.
    // (Also when only the small-tile grid fills the chip and K is very long: 256 x 256 x 65536 x 16
    // fp32 took 1536 us on 256 small tiles and 1083 us split; below 512 K tiles the split's extra
    // pass costs more than it gains -- 2048 x 2048 x 16384 bf16: 130 us against 152 us.)
    const pgk::TileShape big = pgk::mfma_tile_shape(dtype, false);
    const long double big_tiles = (long double)((M + big.bm - 1) / big.bm) * ((N + big.bn - 1) / big.bn) * batch;
    // (skinny tiles run at the speed of their operand stream, which takes two workgroups per CU
    // to keep busy: 16 x 32000 x 4096 fp32, 250 flat tiles, 122 us in one piece and 94 us in two slices)
    const bool skinny = fp.path.kind == pgk::TILE_NARROW || fp.path.kind == pgk::TILE_FLAT;
    // (a bf16 large-tile grid is only chosen from half the CUs' worth of tiles on, and then runs
    // in one piece: two slices of 160 tiles would be a round and a quarter plus the second pass)
    const bool bf16_large = dtype == PGK_DTYPE_BF16 && fp.path.kind == pgk::TILE_LARGE;
    const bool few_tiles = !bf16_large &&
                           (long double)tiles_m * tiles_n * batch < (skinny ? (3 * kNumCUs) / 2 : (3 * kNumCUs) / 4);
    const bool long_k = !bf16_large && big_tiles < (3 * kNumCUs) / 4 && (K + big.bk - 1) / big.bk >= kLongKSteps;
    // (The fp32 small tile fits a CU four times; a grid that fills less than three quarters of
    // those places leaves each CU with one wave per SIMD and nothing to hide its waits behind.
    // From 128 K tiles on the split pays: 16384 x 64 x 8192 275 -> 173 us, 1024 x 1024 x 4096 81 -> 72 us;
    // at 64 K tiles it is even, at 32 it loses.)
    const bool under_filled = dtype == PGK_DTYPE_F32 && fp.path.kind == pgk::TILE_SMALL &&
                              (long double)tiles_m * tiles_n * batch < 3 * kNumCUs && (K + big.bk - 1) / big.bk >= 128;
    if (fp.path.mfma && (few_tiles || long_k || under_filled)) {
        fp.slices = plan_splits(M, N, K, batch, dtype, 0);
        fp.split_small_tile = auto_split(M, N, K, batch, dtype).kind;
        const long double ws_bytes = (long double)batch * fp.slices.splits * M * N * sizeof(float);
        fp.split = fp.slices.splits > 1 && ws_bytes <= (long double)kAutoSplitMaxWorkspace;
    }
    return fp;
}

// ---- The caller's workspace.  Everything a call needs beyond its inputs and outputs is cut from
// it, each piece starting on a multiple of 256 bytes from its (16-byte aligned) base:
//   products  split-K partial products [batch][slices][M][N] fp32 (first, at offset 0)
//   rs_part   row-sum partials, per tile column (single pass) or per column segment (second pass)
//   pack_a/b  zero-padded (or transposed) copies of operands the kernels cannot read in place
// The sizes depend on the shape, the layout of B, whether row sums are wanted and whether A / B
// start on 16-byte boundaries -- the same function answers the workspace queries and lays the
// workspace out inside the calls.
struct WsNeeds {
    bool ok;                 // sizes are representable
    PackDims d;
    bool pack_a, pack_b;
    FusedPlan fp;            // fused call only
    size_t products, rs_part, a_bytes, b_bytes;
    size_t off_rs_part, off_a, off_b, total;
};

void lay_out(WsNeeds& w)
{
    size_t at = round_up256(w.products);
    w.off_rs_part = at; at += round_up256(w.rs_part);
    w.off_a = at; at += round_up256(w.a_bytes);
    w.off_b = at; at += round_up256(w.b_bytes);
    w.total = at;
}

// the operand copies of a packed problem (see pack_dims); a_mis / b_mis: that operand does not
// start on a 16-byte boundary
bool pack_needs(WsNeeds& w, int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, bool b_trans, bool a_mis, bool b_mis)
{
    const size_t es = dtype == PGK_DTYPE_BF16 ? 2 : 4;
    w.d = pack_dims(M, N, K, dtype, b_trans, a_mis || b_mis);
    w.pack_a = w.pack_b = false;
    w.a_bytes = w.b_bytes = 0;
    if (!w.d.pack) return true;
    w.pack_a = w.d.k != K || a_mis;
    w.pack_b = w.d.transpose_b || w.d.k != K || (!b_trans && w.d.ldb != N) || b_mis;
    const int64_t b_rows = w.d.b_trans ? N : w.d.k;
    const long double total = (long double)batch * M * w.d.k * es + (long double)batch * b_rows * w.d.ldb * es;
    if (total >= 4.0e12L) return false;
    if (w.pack_a) w.a_bytes = (size_t)batch * (size_t)M * (size_t)w.d.k * es;
    if (w.pack_b) w.b_bytes = (size_t)batch * (size_t)b_rows * (size_t)w.d.ldb * es;
    return true;
}

WsNeeds fused_needs(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, bool b_trans, bool want_rowsum, bool a_mis,
                    bool b_mis)
{
    WsNeeds w{};
    w.ok = pack_needs(w, M, N, K, batch, dtype, b_trans, a_mis, b_mis);
    if (!w.ok) return w;
    // the problem as the kernels see it
    const bool packed = w.d.pack;
    const int64_t Kc = packed ? w.d.k : K;
    w.fp = plan_fused(packed || !(a_mis || b_mis), M, N, Kc, batch, dtype, packed ? w.d.b_trans : b_trans, packed ? w.d.ldb : 0);
    if (w.fp.split) {
        w.products = (size_t)batch * (size_t)w.fp.slices.splits * (size_t)M * (size_t)N * sizeof(float);
        w.rs_part = split_part_bytes(M, N, batch, want_rowsum);
    } else {
        const int64_t tiles_n = (N + w.fp.path.tile.bn - 1) / w.fp.path.tile.bn;
        if ((long double)batch * tiles_n * M * 4.0L >= 1.8e19L) { w.ok = false; return w; }
        w.rs_part = (want_rowsum && tiles_n > 1) ? (size_t)batch * (size_t)tiles_n * (size_t)M * sizeof(float) : 0;
    }
    lay_out(w);
    return w;
}

WsNeeds splitk_needs(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int effective_splits, bool b_trans,
                     bool want_rowsum, bool a_mis, bool b_mis)
{
    WsNeeds w{};
    w.ok = pack_needs(w, M, N, K, batch, dtype, b_trans, a_mis, b_mis);
    if (!w.ok) return w;
    if ((long double)batch * effective_splits * M * N * sizeof(float) >= 1.8e19L) { w.ok = false; return w; }
    w.products = (size_t)batch * (size_t)effective_splits * (size_t)M * (size_t)N * sizeof(float);
    w.rs_part = split_part_bytes(M, N, batch, want_rowsum);
    lay_out(w);
    return w;
}

bool sizes_valid(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype)
{
    const void* ok = reinterpret_cast<const void*>(uintptr_t{256});
    return validate_common(ok, ok, ok, M, N, K, batch, PGK_ACT_NONE, dtype) == PGK_OK;
}

// Zero-padded copies of the operands of a packed problem (see pack_dims) into the workspace
// pieces w.off_a / w.off_b: A' [batch][M][d.k] when K is ragged or A misaligned, B' [batch][d.k][d.ldb]
// (or Bt' [batch][N][d.k]) when K or its rows are ragged or B misaligned, or when a narrow plain
// B is to be transposed (d.transpose_b; `b_trans` is the layout of the B given).
struct PackedOperands { const void* A; const void* B; };

int pack_operands(const WsNeeds& w, unsigned char* base, const void* A, const void* B, int64_t M, int64_t N, int64_t K,
                  int64_t batch, int dtype, bool b_trans, hipStream_t st, PackedOperands* out)
{
    const PackDims& d = w.d;
    *out = PackedOperands{A, B};
    hipError_t e = hipSuccess;
    if (w.pack_a) {
        unsigned char* p = base + w.off_a;
        e = pgk::launch_pad_matrix(A, p, batch, (int)M, (int)K, (int)M, (int)d.k, dtype, st);
        if (e != hipSuccess) return PGK_ERR_HIP;
        out->A = p;
    }
    if (w.pack_b) {
        unsigned char* p = base + w.off_b;
        e = d.transpose_b ? pgk::launch_transpose_pad(B, p, batch, (int)K, (int)N, (int)d.ldb, dtype, st)
            : b_trans     ? pgk::launch_pad_matrix(B, p, batch, (int)N, (int)K, (int)N, (int)d.k, dtype, st)
                          : pgk::launch_pad_matrix(B, p, batch, (int)K, (int)N, (int)d.k, (int)d.ldb, dtype, st);
        if (e != hipSuccess) return PGK_ERR_HIP;
        out->B = p;
    }
    return PGK_OK;
}

int check_workspace(const WsNeeds& w, const void* workspace, size_t workspace_bytes)
{
    if (!w.ok) return PGK_ERR_UNSUPPORTED;
    if (w.total == 0) return PGK_OK;
    if (!workspace || workspace_bytes < w.total || !aligned16(workspace)) return PGK_ERR_WORKSPACE;
    return PGK_OK;
}

// ---- pgk_gemm_fused_static: the workspace of callers that cannot supply one.  A fixed array in
// the library's device image; each GPU the library runs on holds its own copy, at its own
// address, until the process ends.  Host code never uses the array's name as a pointer: the
// device address is looked up once per device and cached.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
void* g_static_ptr[kMaxDevices] = {};

int static_scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return PGK_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_static_mu);
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PGK_ERR_HIP;
        g_static_ptr[dev] = p;
    }
    *out = g_static_ptr[dev];
    return PGK_OK;
}

// pgk_gemm_fused and pgk_gemm_fused_bt (b_trans: B given as [batch][N][K])
int gemm_fused_impl(const void* A, const void* B, const float* bias, void* C, float* rowsum,
                    int64_t M, int64_t N, int64_t K, int64_t batch, int act, int dtype,
                    void* workspace, size_t workspace_bytes, void* stream, bool b_trans)
{
    int rc = validate_common(A, B, C, M, N, K, batch, act, dtype);
    if (rc != PGK_OK) return rc;
    const bool a_mis = !aligned16(A), b_mis = !aligned16(B);
    const WsNeeds w = fused_needs(M, N, K, batch, dtype, b_trans, rowsum != nullptr, a_mis, b_mis);
    rc = check_workspace(w, workspace, workspace_bytes);
    if (rc != PGK_OK) return rc;
    const FusedPlan& fp = w.fp;
    const Path& path = fp.path;
    const int64_t tiles_m = (M + path.tile.bm - 1) / path.tile.bm;
    const int64_t tiles_n = (N + path.tile.bn - 1) / path.tile.bn;
    if ((long double)tiles_m * tiles_n * batch > 2.0e9L) return PGK_ERR_UNSUPPORTED;
    // ---- everything below enqueues work
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* base = static_cast<unsigned char*>(workspace);
    PackedOperands pk{A, B};
    int64_t ldb = 0;
    bool aligned = !(a_mis || b_mis);
    if (w.d.pack) {
        rc = pack_operands(w, base, A, B, M, N, K, batch, dtype, b_trans, st, &pk);
        if (rc != PGK_OK) return rc;
        K = w.d.k; b_trans = w.d.b_trans; ldb = w.d.ldb;
        aligned = true;
    }
    float* part = w.rs_part ? reinterpret_cast<float*>(base + w.off_rs_part) : nullptr;

    if (fp.split)
        return run_split_passes(pk.A, pk.B, bias, C, rowsum, M, N, K, batch, act, dtype, fp.slices, fp.split_small_tile,
                                reinterpret_cast<float*>(base), part, st, aligned, b_trans, ldb);

    GemmArgs a{};
    a.A = pk.A; a.B = pk.B; a.bias = bias; a.C = C; a.ws = nullptr;
    a.M = (int)M; a.N = (int)N; a.K = (int)K; a.batch = (int)batch;
    pgk::fill_plain_views(a);
    if (b_trans) pgk::set_b_transposed(a);
    if (ldb) set_ldb(a, ldb);
    mark_ragged_rows(a, dtype);
    a.act = act; a.splits = 1;
    a.k_slice = (int)(((K + path.tile.bk - 1) / path.tile.bk) * path.tile.bk);
    a.tiles_m = (int)tiles_m; a.tiles_n = (int)tiles_n;
    a.group_m = group_m_for(a.tiles_m, a.tiles_n);
    // one tile column: the kernel's row sums are final; several: per-tile-column partials, added
    // in tile-column order by a second small kernel
    if (rowsum) a.rs_part = tiles_n == 1 ? rowsum : part;
    if (path.mfma) mark_k_rotation(a, dtype, path.tile);
    hipError_t e = path.mfma ? pgk::launch_gemm_mfma(a, dtype, path.kind, 0, st) : pgk::launch_gemm_guarded(a, dtype, 0, st);
    if (e != hipSuccess) return PGK_ERR_HIP;
    if (rowsum && tiles_n > 1) {
        e = pgk::launch_rowsum_combine(part, rowsum, (int)M, (int)batch, (int)tiles_n, st);
        if (e != hipSuccess) return PGK_ERR_HIP;
    }
    return PGK_OK;
}

}  // namespace

extern "C" {

int pgk_gemm_fused(const void* A, const void* B, const float* bias, void* C, float* rowsum,
                   int64_t M, int64_t N, int64_t K, int64_t batch, int act, int dtype,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    return gemm_fused_impl(A, B, bias, C, rowsum, M, N, K, batch, act, dtype, workspace, workspace_bytes, stream, false);
}

int pgk_gemm_fused_bt(const void* A, const void* Bt, const float* bias, void* C, float* rowsum,
                      int64_t M, int64_t N, int64_t K, int64_t batch, int act, int dtype,
                      void* workspace, size_t workspace_bytes, void* stream)
{
    return gemm_fused_impl(A, Bt, bias, C, rowsum, M, N, K, batch, act, dtype, workspace, workspace_bytes, stream, true);
}

int pgk_gemm_fused_static(const void* A, const void* B, const float* bias, void* C, float* rowsum,
                          int64_t M, int64_t N, int64_t K, int64_t batch, int act, int dtype, void* stream)
{
    int rc = validate_common(A, B, C, M, N, K, batch, act, dtype);
    if (rc != PGK_OK) return rc;
    // the need is known on the host: refuse before touching the device
    const WsNeeds w = fused_needs(M, N, K, batch, dtype, false, rowsum != nullptr, !aligned16(A), !aligned16(B));
    if (!w.ok) return PGK_ERR_UNSUPPORTED;
    if (w.total > kStaticScratchBytes) return PGK_ERR_WORKSPACE;
    void* ws = nullptr;
    if (w.total) {
        rc = static_scratch_of_current_device(&ws);
        if (rc != PGK_OK) return rc;
    }
    return gemm_fused_impl(A, B, bias, C, rowsum, M, N, K, batch, act, dtype, ws, w.total ? kStaticScratchBytes : 0, stream, false);
}

size_t pgk_gemm_fused_static_max_bytes(void) { return kStaticScratchBytes; }

size_t pgk_gemm_fused_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int flags)
{
    if (!sizes_valid(M, N, K, batch, dtype) || (flags & ~(PGK_WS_ROWSUM | PGK_WS_B_TRANSPOSED | PGK_WS_UNALIGNED))) return 0;
    const bool mis = (flags & PGK_WS_UNALIGNED) != 0;
    const WsNeeds w = fused_needs(M, N, K, batch, dtype, (flags & PGK_WS_B_TRANSPOSED) != 0, (flags & PGK_WS_ROWSUM) != 0, mis, mis);
    return w.ok ? w.total : 0;
}

int pgk_gemm_plan(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int b_transposed, int32_t* out)
{
    if (!out) return PGK_ERR_INVALID_ARG;
    const void* ok = reinterpret_cast<const void*>(uintptr_t{256});   // stands for any 16-byte aligned pointer
    const int rc = validate_common(ok, ok, ok, M, N, K, batch, PGK_ACT_NONE, dtype);
    if (rc != PGK_OK) return rc;
    const PackDims d = pack_dims(M, N, K, dtype, b_transposed != 0);      // as pgk_gemm_fused sees the problem
    K = d.k;
    const FusedPlan fp = plan_fused(true, M, N, K, batch, dtype, d.b_trans, d.ldb);
    Path path = fp.path;
    int slices = 1;
    if (fp.split) {
        slices = fp.slices.splits;
        path = choose_path(true, M, N, K, dtype, batch * slices, fp.split_small_tile, d.b_trans, d.ldb);
    }
    const long double wgs = (long double)((M + path.tile.bm - 1) / path.tile.bm) * ((N + path.tile.bn - 1) / path.tile.bn) *
                            batch * slices;
    if (wgs > 2.0e9L) return PGK_ERR_UNSUPPORTED;
    out[0] = path.mfma ? 1 : 0;
    out[1] = path.tile.bm; out[2] = path.tile.bn; out[3] = path.tile.bk;
    out[4] = slices;
    out[5] = (int32_t)wgs;
    return PGK_OK;
}

int pgk_splitk_auto_splits(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int splits)
{
    if (M <= 0 || N <= 0 || K <= 0 || batch <= 0) return 0;
    if (dtype != PGK_DTYPE_F32 && dtype != PGK_DTYPE_BF16) return 0;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim || batch > kMaxDim) return 0;
    if (splits < 0 || splits > K) return 0;
    return plan_splits(M, N, K, batch, dtype, splits).splits;
}

size_t pgk_gemm_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int splits, int flags)
{
    if (!sizes_valid(M, N, K, batch, dtype) || (flags & ~(PGK_WS_ROWSUM | PGK_WS_B_TRANSPOSED | PGK_WS_UNALIGNED))) return 0;
    const int s = pgk_splitk_auto_splits(M, N, K, batch, dtype, splits);
    if (s <= 0) return 0;
    const bool mis = (flags & PGK_WS_UNALIGNED) != 0;
    const WsNeeds w = splitk_needs(M, N, K, batch, dtype, s, (flags & PGK_WS_B_TRANSPOSED) != 0, (flags & PGK_WS_ROWSUM) != 0, mis, mis);
    return w.ok ? w.total : 0;
}

size_t pgk_splitk_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t batch, int dtype, int splits)
{
    // enough for either layout of B, with or without row sums, operands on 16-byte boundaries
    const size_t plain = pgk_gemm_splitk_workspace_bytes(M, N, K, batch, dtype, splits, PGK_WS_ROWSUM);
    const size_t bt = pgk_gemm_splitk_workspace_bytes(M, N, K, batch, dtype, splits, PGK_WS_ROWSUM | PGK_WS_B_TRANSPOSED);
    return plain > bt ? plain : bt;
}

}  // extern "C"

namespace {

int gemm_splitk_impl(const void* A, const void* B, const float* bias, void* C, float* rowsum,
                     int64_t M, int64_t N, int64_t K, int64_t batch, int act, int dtype, int splits,
                     void* workspace, size_t workspace_bytes, void* stream, bool b_trans)
{
    int rc = validate_common(A, B, C, M, N, K, batch, act, dtype);
    if (rc != PGK_OK) return rc;
    if (splits < 0 || splits > K) return PGK_ERR_INVALID_ARG;
    const SplitPlan plan = plan_splits(M, N, K, batch, dtype, splits);
    const bool a_mis = !aligned16(A), b_mis = !aligned16(B);
    const WsNeeds w = splitk_needs(M, N, K, batch, dtype, plan.splits, b_trans, rowsum != nullptr, a_mis, b_mis);
    if (!w.ok) return PGK_ERR_UNSUPPORTED;
    rc = check_workspace(w, workspace, workspace_bytes);
    if (rc != PGK_OK) return rc;
    // ---- everything below enqueues work
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* base = static_cast<unsigned char*>(workspace);
    float* part = w.rs_part ? reinterpret_cast<float*>(base + w.off_rs_part) : nullptr;
    // an automatic plan comes with its tile; explicit splits get the tile their grid suggests
    const int small_tile = (splits == 0 && mfma_route(M, N, K, dtype)) ? auto_split(M, N, K, batch, dtype).kind : -1;
    // (the slices are counted in K steps, which padding K to whole chunks leaves as they are)
    if (!w.d.pack)
        return run_split_passes(A, B, bias, C, rowsum, M, N, K, batch, act, dtype, plan, small_tile,
                                reinterpret_cast<float*>(base), part, st, !(a_mis || b_mis), b_trans);
    PackedOperands pk{};
    rc = pack_operands(w, base, A, B, M, N, K, batch, dtype, b_trans, st, &pk);
    if (rc != PGK_OK) return rc;
    return run_split_passes(pk.A, pk.B, bias, C, rowsum, M, N, w.d.k, batch, act, dtype, plan, small_tile,
                            reinterpret_cast<float*>(base), part, st, true, w.d.b_trans, w.d.ldb);
}

}  // namespace

extern "C" {

int pgk_gemm_splitk(const void* A, const void* B, const float* bias, void* C, float* rowsum,
                    int64_t M, int64_t N, int64_t K, int64_t batch, int act, int dtype, int splits,
                    void* workspace, size_t workspace_bytes, void* stream)
{
    return gemm_splitk_impl(A, B, bias, C, rowsum, M, N, K, batch, act, dtype, splits, workspace, workspace_bytes,
                            stream, false);
}

int pgk_gemm_splitk_bt(const void* A, const void* Bt, const float* bias, void* C, float* rowsum,
                       int64_t M, int64_t N, int64_t K, int64_t batch, int act, int dtype, int splits,
                       void* workspace, size_t workspace_bytes, void* stream)
{
    return gemm_splitk_impl(A, Bt, bias, C, rowsum, M, N, K, batch, act, dtype, splits, workspace, workspace_bytes,
                            stream, true);
}

size_t pgk_reduce_max_workspace_bytes(int64_t outer, int64_t red, int64_t inner, int dtype)
{
    if (outer <= 0 || red <= 0 || inner <= 0 || (dtype != PGK_DTYPE_F32 && dtype != PGK_DTYPE_BF16)) return 0;
    if (red > (1LL << 31) - 1024) return 0;
    if ((long double)outer * (long double)inner >= 4.6e18L ||
        (long double)outer * (long double)inner * (long double)red >= 4.6e18L) return 0;
    // (the plan depends on whether X starts on a 16-byte boundary: enough for either case)
    const size_t a = pgk::plan_reduce_max(outer, red, inner, dtype, true).partial_elems;
    const size_t b = pgk::plan_reduce_max(outer, red, inner, dtype, false).partial_elems;
    return (a > b ? a : b) * 8;
}

int pgk_reduce_max(const void* X, void* out, int32_t* idx, int64_t outer, int64_t red, int64_t inner,
                   int dtype, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!X || !out || outer <= 0 || red <= 0 || inner <= 0) return PGK_ERR_INVALID_ARG;
    if (dtype != PGK_DTYPE_F32 && dtype != PGK_DTYPE_BF16) return PGK_ERR_INVALID_ARG;
    if (red > (1LL << 31) - 1024) return PGK_ERR_UNSUPPORTED;
    if ((long double)outer * (long double)inner >= 4.6e18L ||
        (long double)outer * (long double)inner * (long double)red >= 4.6e18L) return PGK_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const pgk::ReducePlan pl = pgk::plan_reduce_max(outer, red, inner, dtype, aligned16(X));
    if (pl.blocks <= 0 || pl.blocks > 0x7fffffffLL) return PGK_ERR_UNSUPPORTED;
    float* pv = nullptr;
    int* pi = nullptr;
    if (pl.partial_elems) {
        // segment results (value, position) of the first pass
        if (!workspace || workspace_bytes < pl.partial_elems * 8 || (reinterpret_cast<uintptr_t>(workspace) & 3u))
            return PGK_ERR_WORKSPACE;
        pv = static_cast<float*>(workspace);
        pi = reinterpret_cast<int*>(pv + pl.partial_elems);
    }
    const hipError_t e = pgk::launch_reduce_max(pl, X, out, idx, pv, pi, outer, red, inner, dtype, st);
    return e == hipSuccess ? PGK_OK : PGK_ERR_HIP;
}

}  // extern "C"

namespace {

struct ConvPlan {
    bool valid;          // arguments make sense
    bool fast;           // matrix-core path
    int64_t Lout;
    // matrix-core path, where the B operand comes from:
    //   strips: the input itself; the tile columns whose reads would leave a row (listed in
    //           edge_tn) read zero-padded strips of edge_w columns instead;
    //   table:  stride * shifts copies of the input (see launch_conv_phase_copies), rows of Lq
    //           elements and cin_pad channels; tap k reads copy (k dil mod stride, h) at column
    //           offset (k dil div stride) - h, with h = 1 where that offset would be odd in bf16;
    //   else:   a zero-padded copy of the whole input with rows of Lp elements (Lp = 0: the
    //           input as it is -- no padding and aligned rows)
    bool strips;
    int n_edges;
    int edge_tn[3];
    int edge_first_col[3];
    int64_t edge_w;
    int64_t Lp;
    bool table;
    int shifts;
    int64_t Lq, cin_pad;
    int kind;            // tile shape (TILE_*), chosen as for a plain GEMM of Cout x Lout
    pgk::TileShape tile;
    size_t w_bytes, x_bytes;   // workspace parts: regrouped weights; copies of the input or strips
};

size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

ConvPlan plan_conv1d(int64_t B, int64_t Cin, int64_t L, int64_t Cout, int64_t Kw, int64_t stride, int64_t pad,
                     int64_t dilation, int dtype)
{
    ConvPlan pl{};
    if (B <= 0 || Cin <= 0 || L <= 0 || Cout <= 0 || Kw <= 0 || stride <= 0 || pad < 0 || dilation <= 0) return pl;
    if (dtype != PGK_DTYPE_F32 && dtype != PGK_DTYPE_BF16) return pl;
    if (B > kMaxDim || Cin > kMaxDim || L > kMaxDim || Cout > kMaxDim || Kw > kMaxDim || pad > kMaxDim ||
        dilation > kMaxDim || stride > kMaxDim) return pl;
    const int64_t span = L + 2 * pad - dilation * (Kw - 1) - 1;
    if (span < 0) return pl;
    pl.Lout = span / stride + 1;
    if (Cin * Kw > kMaxDim) return pl;
    pl.valid = true;
    const int64_t es = dtype == PGK_DTYPE_BF16 ? 2 : 4, epc = 16 / es;
    const pgk::TileShape t = pgk::mfma_tile_shape(dtype, false);
    // very short outputs stay with the bounds-checked kernel.  The output length may be anything
    // (the kernels store a row's last, partly filled chunk element by element), but the B copies
    // then reach up to Lr - 1 = the last column of that chunk, which the copies of the input must hold.
    if (pl.Lout < 16) return pl;
    const int64_t Lr = (int64_t)round_up((size_t)pl.Lout, (size_t)epc);
    // (up to 32 output channels: the flat tile, as for a GEMM with that many rows)
    pl.kind = Cout <= 32 ? pgk::TILE_FLAT : auto_tile_kind(Cout, pl.Lout, 0, dtype, B, false);
    pl.tile = pgk::mfma_tile_shape(dtype, pl.kind);
    const int64_t bn = pl.tile.bn, halo = (Kw - 1) * dilation;
    const bool shifts_even = dtype == PGK_DTYPE_F32 || dilation % 2 == 0 || Kw == 1;

    if (stride == 1 && Cin % t.bk == 0 && shifts_even) {
        // the input as it is, or one zero-padded copy of it; taps a constant column step apart
        const int64_t K = Cin * Kw;
        const bool needs_copy = pad > 0 || L % epc != 0 || pl.Lout % epc != 0;
        const int64_t Lp = needs_copy ? (int64_t)round_up((size_t)std::max(L + 2 * pad, Lr + halo), (size_t)epc) : L;
        if ((int64_t)t.bm * K * es >= (1LL << 32) || (int64_t)t.bk * Lp * es + dilation * Kw * es >= (1LL << 32)) return pl;
        pl.fast = true;
        pl.w_bytes = round_up((size_t)(Cout * K * es), 256);
        // Reading the input in place needs every tile base 4-byte aligned (rows and shifts), the
        // halo and the padding no wider than a tile.
        pl.strips = pl.Lout % epc == 0 && halo <= bn && pad <= bn && (L * es) % 4 == 0 && (pad * es) % 4 == 0 &&
                    (long double)B * Cin * 3 * ((bn + halo) / 256 + 2) < 2.0e9L;
        if (pl.strips) {
            const int64_t tiles_n = (pl.Lout + bn - 1) / bn;
            pl.edge_w = (int64_t)round_up((size_t)(bn + halo), (size_t)epc);
            pl.n_edges = 0;
            if (pad > 0) {
                const int64_t r0 = pl.Lout > pad ? (pl.Lout - pad) / bn : 0;     // first tile column reading past the end
                for (int64_t tn = 0; tn < tiles_n; ++tn)
                    if (tn == 0 || tn >= r0) {
                        pl.edge_tn[pl.n_edges] = (int)tn;
                        pl.edge_first_col[pl.n_edges] = (int)(tn * bn - pad);
                        ++pl.n_edges;
                    }
            }
            pl.x_bytes = round_up((size_t)pl.n_edges * (size_t)B * (size_t)Cin * (size_t)pl.edge_w * (size_t)es, 256);
            pl.Lp = 0;
        } else {
            pl.Lp = needs_copy ? Lp : 0;
            pl.x_bytes = needs_copy ? round_up((size_t)B * (size_t)Cin * (size_t)Lp * (size_t)es, 256) : 0;
        }
        return pl;
    }

    // Everything else with enough channels: stride > 1 (one copy per phase), a channel count
    // that is not a multiple of the K tile (copies and weights padded with zero channels), bf16
    // taps at odd column offsets (a second copy shifted by one element).  Each tap's place comes
    // from a table.  Padding the channels more than twofold would cost more than it gains.
    pl.cin_pad = (int64_t)round_up((size_t)Cin, (size_t)t.bk);
    if (Kw > pgk::kMaxTableTaps || pl.cin_pad > 2 * Cin) return pl;
    const int64_t K = pl.cin_pad * Kw;
    const int64_t q_max = halo / stride;
    pl.shifts = 1;
    if (dtype == PGK_DTYPE_BF16)
        for (int64_t k = 0; k < Kw; ++k)
            if ((k * dilation / stride) % 2 != 0) pl.shifts = 2;
    pl.Lq = (int64_t)round_up((size_t)(Lr + q_max + 1), (size_t)epc);
    if ((int64_t)t.bm * K * es >= (1LL << 32) || (int64_t)t.bk * pl.Lq * es >= (1LL << 32)) return pl;
    const long double copies_bytes = (long double)stride * pl.shifts * B * pl.cin_pad * pl.Lq * es;
    if (copies_bytes >= 4.0e12L || (long double)stride * pl.shifts * B * pl.cin_pad > 4.0e9L) return pl;
    pl.fast = true;
    pl.table = true;
    pl.w_bytes = round_up((size_t)(Cout * K * es), 256);
    pl.x_bytes = round_up((size_t)copies_bytes, 256);
    return pl;
}

}  // namespace

extern "C" {

int64_t pgk_conv1d_out_len(int64_t L, int64_t Kw, int64_t stride, int64_t pad, int64_t dilation)
{
    if (L <= 0 || Kw <= 0 || stride <= 0 || pad < 0 || dilation <= 0) return 0;
    const int64_t span = L + 2 * pad - dilation * (Kw - 1) - 1;
    return span < 0 ? 0 : span / stride + 1;
}

size_t pgk_conv1d_workspace_bytes(int64_t B, int64_t Cin, int64_t L, int64_t Cout, int64_t Kw, int64_t stride,
                                  int64_t pad, int64_t dilation, int dtype)
{
    const ConvPlan pl = plan_conv1d(B, Cin, L, Cout, Kw, stride, pad, dilation, dtype);
    return (pl.valid && pl.fast) ? pl.w_bytes + pl.x_bytes : 0;
}

int pgk_conv1d(const void* x, const void* w, const float* bias, void* y, int64_t B, int64_t Cin, int64_t L,
               int64_t Cout, int64_t Kw, int64_t stride, int64_t pad, int64_t dilation, int act, int dtype,
               void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !w || !y) return PGK_ERR_INVALID_ARG;
    if (act < PGK_ACT_NONE || act > PGK_ACT_SILU) return PGK_ERR_INVALID_ARG;
    ConvPlan pl = plan_conv1d(B, Cin, L, Cout, Kw, stride, pad, dilation, dtype);
    if (!pl.valid) {
        // tell "out of range" from "makes no sense"
        if (B > 0 && Cin > 0 && L > 0 && Cout > 0 && Kw > 0 && stride > 0 && pad >= 0 && dilation > 0 &&
            (dtype == PGK_DTYPE_F32 || dtype == PGK_DTYPE_BF16) && pgk_conv1d_out_len(L, Kw, stride, pad, dilation) > 0)
            return PGK_ERR_UNSUPPORTED;
        return PGK_ERR_INVALID_ARG;
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t es = dtype == PGK_DTYPE_BF16 ? 2 : 4;
    if ((long double)B * Cout * pl.Lout >= 4.6e18L || (long double)B * Cin * L >= 4.6e18L) return PGK_ERR_UNSUPPORTED;
    // The weights are always regrouped into the workspace, y and the bias may start on any element;
    // only an input that the kernels read in place has to start on a 16-byte boundary.
    const bool reads_x_in_place = pl.strips || (!pl.table && pl.Lp == 0);
    if (pl.fast && reads_x_in_place && !aligned16(x)) pl.fast = false;

    GemmArgs a{};
    a.bias = bias; a.C = y; a.ws = nullptr; a.rs_part = nullptr;
    a.M = (int)Cout; a.N = (int)pl.Lout; a.K = (int)(Cin * Kw); a.batch = (int)B;
    pgk::fill_plain_views(a);
    a.a_batch_stride = 0;                 // the weights are shared by the batch entries
    a.bias_per_row = 1;                   // one bias per output channel = per row
    a.act = act; a.splits = 1;

    if (pl.fast) {
        if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < pl.w_bytes + pl.x_bytes)
            return PGK_ERR_WORKSPACE;
        unsigned char* wr = static_cast<unsigned char*>(workspace);
        unsigned char* xp = wr + pl.w_bytes;
        const void* bsrc = x;
        int64_t ldb = L, cin_k = Cin;
        if (pl.table) {
            cin_k = pl.cin_pad;
            // the copies of the input and the regrouped, channel-padded weights in one launch
            if (pgk::launch_conv_phase_copies(x, xp, B, (int)Cin, (int)pl.cin_pad, (int)L, (int)pl.Lq, (int)pad, (int)stride,
                                              pl.shifts, w, wr, (int)Cout, (int)Kw, dtype, st) != hipSuccess) return PGK_ERR_HIP;
            bsrc = xp;
            ldb = pl.Lq;
            a.K = (int)(pl.cin_pad * Kw);
            a.b_use_tap_table = 1;
            const int64_t plane = B * pl.cin_pad * pl.Lq;          // elements of one copy
            for (int64_t k = 0; k < Kw; ++k) {
                const int64_t o = k * dilation, phase = o % stride, q = o / stride;
                const int64_t h = (pl.shifts == 2 && q % 2 != 0) ? 1 : 0;
                a.b_tap_off[k] = ((phase * pl.shifts + h) * plane + (q - h)) * es;
            }
        } else if (pl.strips) {
            // strips and regrouped weights in one launch
            if (pgk::launch_conv_prepare(x, xp, B * Cin, (int)L, (int)pl.edge_w, pl.n_edges, pl.edge_first_col, w, wr,
                                         (int)Cout, (int)Cin, (int)Kw, dtype, st) != hipSuccess) return PGK_ERR_HIP;
            if (pl.n_edges > 0) {
                for (int e = 0; e < pl.n_edges; ++e) {
                    a.edge_tn[e] = pl.edge_tn[e];
                    a.edge_B[e] = xp + (size_t)e * (size_t)(B * Cin) * (size_t)pl.edge_w * (size_t)es;
                }
                a.edge_ldb = (int)pl.edge_w;
                a.edge_batch_stride = Cin * pl.edge_w;
            }
            a.b_col_shift = -(int)pad;
        } else {
            if (pgk::launch_conv_repack_weights(w, wr, (int)Cout, (int)Cin, (int)Cin, (int)Kw, dtype, st) != hipSuccess)
                return PGK_ERR_HIP;
            if (pl.Lp) {
                if (pgk::launch_conv_pad_input(x, xp, B * Cin, (int)L, (int)pl.Lp, (int)pad, dtype, st) != hipSuccess)
                    return PGK_ERR_HIP;
                bsrc = xp;
                ldb = pl.Lp;
            }
        }
        const Path path = choose_path(aligned16(wr) && aligned16(bsrc), Cout, pl.Lout, cin_k * Kw, dtype, B, pl.kind, false, ldb);
        if (!path.mfma) return PGK_ERR_UNSUPPORTED;   // the plan has checked what the kernel needs
        a.A = wr; a.B = bsrc;
        a.a_batch_stride = 0;
        a.b_batch_stride = cin_k * ldb;
        a.ldb = (int)ldb;
        a.b_tiles_per_tap = (int)(cin_k / path.tile.bk);
        a.b_tap_step = (int)dilation;
        a.k_slice = a.K;
        a.tiles_m = (int)((Cout + path.tile.bm - 1) / path.tile.bm);
        a.tiles_n = (int)((pl.Lout + path.tile.bn - 1) / path.tile.bn);
        if ((long double)a.tiles_m * a.tiles_n * B > 2.0e9L) return PGK_ERR_UNSUPPORTED;
        a.group_m = group_m_for(a.tiles_m, a.tiles_n);
        return pgk::launch_gemm_mfma(a, dtype, path.kind, 0, st) == hipSuccess ? PGK_OK : PGK_ERR_HIP;
    }
    // bounds-checked kernel, input read in place
    const pgk::TileShape t = pgk::guarded_tile_shape();
    a.A = w; a.B = x;
    a.b_batch_stride = Cin * L;
    a.conv_kw = (int)Kw; a.conv_stride = (int)stride; a.conv_pad = (int)pad; a.conv_dil = (int)dilation; a.conv_len = (int)L;
    a.k_slice = (int)(((a.K + t.bk - 1) / t.bk) * t.bk);
    a.tiles_m = (int)((Cout + t.bm - 1) / t.bm);
    a.tiles_n = (int)((pl.Lout + t.bn - 1) / t.bn);
    if ((long double)a.tiles_m * a.tiles_n * B > 2.0e9L) return PGK_ERR_UNSUPPORTED;
    a.group_m = group_m_for(a.tiles_m, a.tiles_n);
    return pgk::launch_gemm_guarded(a, dtype, 0, st) == hipSuccess ? PGK_OK : PGK_ERR_HIP;
}

int pgk_probe_mfma(int dtype, int random_operands, int iters, float* sink, double* flops_out, void* stream)
{
    if (!sink || iters < 1 || iters > (1 << 20)) return PGK_ERR_INVALID_ARG;
    if (dtype != PGK_DTYPE_F32 && dtype != PGK_DTYPE_BF16) return PGK_ERR_INVALID_ARG;
    const int workgroups = 2 * kNumCUs;
    if (flops_out) {
        const double per_instruction = dtype == PGK_DTYPE_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
        *flops_out = per_instruction * 32.0 * iters * 4.0 * workgroups;
    }
    const hipError_t e = pgk::launch_probe_mfma(dtype, random_operands != 0, iters, workgroups, sink,
                                                static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PGK_OK : PGK_ERR_HIP;
}

int pgk_probe_mfma_fed(int copies, int iters, const void* src, size_t src_bytes, size_t resident_bytes,
                       int stream_every, uint64_t* clock_out, double* flops_out, void* stream)
{
    if (!clock_out || (reinterpret_cast<uintptr_t>(clock_out) & 7u)) return PGK_ERR_INVALID_ARG;
    if (iters < 2 || iters > (1 << 20) || (iters & 1) || stream_every < 0) return PGK_ERR_INVALID_ARG;
    const size_t piece = 65536;
    unsigned int resident = 1, streamed = 0;
    if (copies) {
        if (!src || !aligned16(src) || src_bytes < piece || src_bytes % piece != 0) return PGK_ERR_INVALID_ARG;
        if (resident_bytes < piece || resident_bytes % piece != 0 || resident_bytes > src_bytes) return PGK_ERR_INVALID_ARG;
        if (src_bytes / piece > 0x7fffffffu) return PGK_ERR_UNSUPPORTED;
        resident = (unsigned int)(resident_bytes / piece);
        streamed = (unsigned int)((src_bytes - resident_bytes) / piece);
    }
    if (flops_out) *flops_out = 2.0 * 32 * 32 * 16 * 32.0 * iters * 8.0 * kNumCUs;
    const hipError_t e = pgk::launch_probe_mfma_fed(copies != 0, iters, src, resident, streamed, stream_every,
                                                    reinterpret_cast<unsigned long long*>(clock_out),
                                                    static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PGK_OK : PGK_ERR_HIP;
}

int pgk_probe_gemm_phases(const void* A, const void* B, const float* bias, void* C, float* rowsum_partials,
                          int64_t M, int64_t N, int64_t K, int act, int dtype, uint64_t* stamps, size_t stamps_bytes,
                          int32_t* workgroups_out, void* stream)
{
    int rc = validate_common(A, B, C, M, N, K, 1, act, dtype);
    if (rc != PGK_OK) return rc;
    if (!stamps || (reinterpret_cast<uintptr_t>(stamps) & 7u)) return PGK_ERR_INVALID_ARG;
    const pgk::TileShape t = pgk::mfma_tile_shape(dtype, pgk::TILE_LARGE);
    if (!aligned16(A) || !aligned16(B) || !mfma_shape_ok(M, N, K, dtype) || needs_packing(N, K, dtype, false))
        return PGK_ERR_UNSUPPORTED;
    const int64_t tiles_m = (M + t.bm - 1) / t.bm, tiles_n = (N + t.bn - 1) / t.bn;
    if ((long double)tiles_m * tiles_n > 1.0e6L) return PGK_ERR_UNSUPPORTED;
    if (workgroups_out) *workgroups_out = (int32_t)(tiles_m * tiles_n);
    if (stamps_bytes < (size_t)(tiles_m * tiles_n) * pgk::kStampWords * sizeof(uint64_t)) return PGK_ERR_WORKSPACE;
    GemmArgs a{};
    a.A = A; a.B = B; a.bias = bias; a.C = C; a.rs_part = rowsum_partials;
    a.M = (int)M; a.N = (int)N; a.K = (int)K; a.batch = 1;
    pgk::fill_plain_views(a);
    mark_ragged_rows(a, dtype);
    a.act = act; a.splits = 1;
    a.k_slice = (int)(((K + t.bk - 1) / t.bk) * t.bk);
    a.tiles_m = (int)tiles_m; a.tiles_n = (int)tiles_n;
    a.group_m = group_m_for(a.tiles_m, a.tiles_n);
    a.stamps = reinterpret_cast<unsigned long long*>(stamps);
    return pgk::launch_gemm_mfma_timed(a, dtype, static_cast<hipStream_t>(stream)) == hipSuccess ? PGK_OK : PGK_ERR_HIP;
}

int pgk_probe_stream_read(const void* src, size_t bytes, float* sink, void* stream)
{
    if (!src || !sink || bytes == 0 || bytes % 16 || !aligned16(src)) return PGK_ERR_INVALID_ARG;
    const hipError_t e = pgk::launch_probe_stream_read(src, bytes, sink, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PGK_OK : PGK_ERR_HIP;
}

const char* pgk_status_string(int status)
{
    switch (status) {
    case PGK_OK: return "PGK_OK";
    case PGK_ERR_INVALID_ARG: return "PGK_ERR_INVALID_ARG: null pointer, non-positive size, or unknown act/dtype/splits";
    case PGK_ERR_UNSUPPORTED: return "PGK_ERR_UNSUPPORTED: size beyond the supported index range";
    case PGK_ERR_WORKSPACE: return "PGK_ERR_WORKSPACE: workspace missing, misaligned or too small";
    case PGK_ERR_HIP: return "PGK_ERR_HIP: the HIP runtime reported an error";
    default: return "PGK: unknown status";
    }
}

int pgk_version(void) { return 200; }

}  // extern "C"
