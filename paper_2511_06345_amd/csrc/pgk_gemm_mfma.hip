// Matrix-core GEMM main loop with the fused epilogue, for gfx950 (MI355X).
//
// The operator is the textbook one the paper's matmul / activation / reduction
// categories refer to (PRAGMA Sections 1 and 4.2): C = act(A*B + bias) with an
// optional row sum.  Everything about how it is computed below is this
// library's own design for CDNA4:
//
//  * One workgroup owns a BM x BN tile of C.  A and B tiles of BK along K are
//    copied global -> LDS with 128-bit direct-to-LDS loads into a two-stage
//    ring, so the copy of tile kt+1 overlaps the matrix-core work on tile kt.
//  * LDS rows are stored in 16-byte chunks whose position is XOR-swizzled with
//    the row index; the direct-to-LDS write is always one contiguous 1 KiB per
//    wave instruction, so the swizzle is applied by choosing which global chunk
//    each lane fetches.
//  * MFMA operand roles are swapped (the B-matrix columns feed the "A" operand
//    and the A-matrix rows the "B" operand), so the accumulator tile a lane holds
//    is one row of C with runs of 4 consecutive columns.  Row sums are then
//    mostly in-lane adds, bias loads and C stores are 4 elements wide.
//  * bf16: v_mfma_f32_32x32x16_bf16.  A rows are K-contiguous in LDS
//    (ds_read_b128); B is N-contiguous, so its operand is gathered with the
//    transposing ds_read_b64_tr_b16.
//  * fp32: v_mfma_f32_32x32x2_f32.
//  * Workgroup ids are remapped so that each XCD (own L2) works on a compact
//    group of tiles.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "pgk_device.h"
#include "pgk_kernels.h"

namespace pgk {

template <bool BF16_, int BM_, int BN_, int BK_, int WGM_, int WGN_, int COPY_PARTS_, int STAGES_ = 2,
          int WAVES_PER_SIMD_ = 1>
struct MfmaCfg {
    // depth of the LDS ring of K tiles (2..5): STAGES - 1 tiles are in flight or landed
    // ahead of the one being multiplied
    static constexpr int STAGES = STAGES_;
    // waves the register allocation must leave room for on one SIMD
    static constexpr int WAVES_PER_SIMD = WAVES_PER_SIMD_;
    // The global -> LDS copy of one K tile is issued in COPY_PARTS_ equal parts, one
    // part per operand-fetch step, so that the texture-address path (16 cycles per
    // 1 KiB wave instruction) is never asked for more than it can take in a step.
    static constexpr int COPY_PARTS = COPY_PARTS_;
    static constexpr bool BF16 = BF16_;
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
    static constexpr int ES = BF16_ ? 2 : 4;       // element bytes
    static constexpr int NW = WGM * WGN;           // waves per workgroup
    static constexpr int NT = NW * 64;             // threads per workgroup
    static constexpr int WM = BM / WGM;            // rows per wave
    static constexpr int WN = BN / WGN;            // cols per wave
    static constexpr int TM = WM / 32, TN = WN / 32;
    static constexpr int RA = BK * ES;             // LDS row bytes of the A tile
    static constexpr int RB = BN * ES;             // LDS row bytes of the B tile
    static constexpr int A_BYTES = BM * RA, B_BYTES = BK * RB;
    static constexpr int A_CPW = A_BYTES / 1024 / NW;  // 1 KiB chunks per wave
    static constexpr int B_CPW = B_BYTES / 1024 / NW;
    static constexpr int A_CPR = RA / 16, B_CPR = RB / 16;  // 16 B chunks per row
    static constexpr int A_RPC = 1024 / RA, B_RPC = 1024 / RB;  // rows per 1 KiB
    static constexpr int LDS_BYTES = STAGES * (A_BYTES + B_BYTES);
    static_assert(STAGES >= 2 && STAGES <= 5 && LDS_BYTES <= 160 * 1024, "LDS ring size");
    static_assert(RA == 128 || RA == 64, "A-tile swizzle assumes 128- or 64-byte rows");
    static_assert(RB % 256 == 0, "B-tile swizzle assumes rows of a multiple of 256 bytes");
    static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile / wave split");
    static_assert(BM <= NT, "row-sum combine uses one thread per tile row");
};

// Swizzles (in units of 16-byte chunks) applied to the chunk index of a row.
// A tile: rows of CPR chunks; 16 consecutive rows read the same logical chunk
// at once, so the 16 chunk slots of a 256-byte bank period must all differ.
template <int CPR>
__device__ __forceinline__ int swz_a(int row) { return (row / (16 / CPR)) % CPR; }
template <bool BF16>
__device__ __forceinline__ int swz_b(int krow)
{
    // bf16: the transposing read of a 16-lane group touches 4 consecutive k rows;
    // fp32: the two half-waves read rows 4 apart.
    return BF16 ? 4 * (krow & 3) : 8 * ((krow >> 2) & 1);
}

template <int ACT, bool OUT_BF16, int TM, int TN>
__device__ __forceinline__ void epilogue_fused(f32x16 (&acc)[TM][TN], const GemmArgs& p,
                                               size_t c_base, int m_wave, int n_wave, int lane,
                                               float* rs_lds)
{
    const int half = lane >> 5;
    const int row_in = lane & 31;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        float rs = 0.0f;
        const size_t row_off = c_base + (size_t)(m_wave + 32 * i + row_in) * (size_t)p.N;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n_wave + 32 * j + 8 * g + 4 * half;
                f32x4 bv = {0.f, 0.f, 0.f, 0.f};
                if (p.bias) bv = *(const f32x4*)(p.bias + n);
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    y[e] = activate<ACT>(acc[i][j][4 * g + e] + bv[e]);
                    rs += y[e];
                }
                if constexpr (OUT_BF16) {
                    u32x2 pk = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
                    *(u32x2*)((unsigned short*)p.C + row_off + n) = pk;
                } else {
                    f32x4 o = {y[0], y[1], y[2], y[3]};
                    *(f32x4*)((float*)p.C + row_off + n) = o;
                }
            }
        }
        if (rs_lds) {
            rs += __shfl_xor(rs, 32);
            if (half == 0) rs_lds[32 * i + row_in] = rs;
        }
    }
}

template <int V>
struct IC { static constexpr int value = V; };

template <typename Cfg>
__global__ __launch_bounds__(Cfg::NT, Cfg::WAVES_PER_SIMD) void gemm_mfma_kernel(const GemmArgs p, const int out_mode)
{
    constexpr bool BF16 = Cfg::BF16;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, ES = Cfg::ES;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, RA = Cfg::RA, RB = Cfg::RB;
    constexpr int NS = BF16 ? BK / 16 : BK / 8;   // operand-fetch steps per K tile
    static_assert(NS % 2 == 0, "fragment double buffer assumes an even step count");

    // Separate LDS objects per stage and operand (not one array indexed by stage): the
    // compiler can then tell that a direct-to-LDS copy into one stage does not alias
    // the operand reads of another stage, and does not wait for it.
    constexpr int S = Cfg::STAGES;
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a0[Cfg::A_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a1[Cfg::A_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a2[S > 2 ? Cfg::A_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a3[S > 3 ? Cfg::A_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_a4[S > 4 ? Cfg::A_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_b0[Cfg::B_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_b1[Cfg::B_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_b2[S > 2 ? Cfg::B_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_b3[S > 3 ? Cfg::B_BYTES : 16];
    __shared__ __attribute__((aligned(1024))) unsigned char lds_b4[S > 4 ? Cfg::B_BYTES : 16];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / Cfg::WGN, wn = wave % Cfg::WGN;

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
    const int KT = (k_end - k_begin) / BK;

    const unsigned char* Ag = (const unsigned char*)p.A +
        ((size_t)b * p.M * p.K + (size_t)tm * BM * p.K + (size_t)k_begin) * ES;
    const unsigned char* Bg = (const unsigned char*)p.B +
        ((size_t)b * p.K * p.N + (size_t)k_begin * p.N + (size_t)tn * BN) * ES;
    const size_t a_step = (size_t)BK * ES;             // bytes per K tile along an A row
    const size_t b_step = (size_t)BK * p.N * ES;       // bytes per K tile down B

    // ---- per-lane byte offsets of the global chunks this lane copies
    unsigned int voff_a[Cfg::A_CPW], voff_b[Cfg::B_CPW];
#pragma unroll
    for (int t = 0; t < Cfg::A_CPW; ++t) {
        const int ch = wave * Cfg::A_CPW + t;
        const int r = ch * Cfg::A_RPC + lane / Cfg::A_CPR;
        const int c = (lane % Cfg::A_CPR) ^ swz_a<Cfg::A_CPR>(r);
        voff_a[t] = (unsigned int)r * (unsigned int)p.K * ES + (unsigned int)c * 16u;
    }
#pragma unroll
    for (int t = 0; t < Cfg::B_CPW; ++t) {
        const int ch = wave * Cfg::B_CPW + t;
        const int kr = ch * Cfg::B_RPC + lane / Cfg::B_CPR;
        const int c = (lane % Cfg::B_CPR) ^ swz_b<BF16>(kr);
        voff_b[t] = (unsigned int)kr * (unsigned int)p.N * ES + (unsigned int)c * 16u;
    }

    auto lds_a = [&](auto st) -> unsigned char* {
        constexpr int v = decltype(st)::value;
        if constexpr (v == 0) return lds_a0; else if constexpr (v == 1) return lds_a1;
        else if constexpr (v == 2) return lds_a2; else if constexpr (v == 3) return lds_a3; else return lds_a4;
    };
    auto lds_b = [&](auto st) -> unsigned char* {
        constexpr int v = decltype(st)::value;
        if constexpr (v == 0) return lds_b0; else if constexpr (v == 1) return lds_b1;
        else if constexpr (v == 2) return lds_b2; else if constexpr (v == 3) return lds_b3; else return lds_b4;
    };

    // global -> LDS copy of K tile kt into stage st: instructions of part `part`
    // (the A and B instructions of a wave are numbered together, A first)
    constexpr int N_COPY = Cfg::A_CPW + Cfg::B_CPW;
    constexpr int PER_PART = (N_COPY + Cfg::COPY_PARTS - 1) / Cfg::COPY_PARTS;
    auto load_part = [&](int kt, auto st, int part) {
        const unsigned char* ga = Ag + (size_t)kt * a_step;
        const unsigned char* gb = Bg + (size_t)kt * b_step;
        unsigned char* la = lds_a(st) + wave * (Cfg::A_CPW * 1024);
        unsigned char* lb = lds_b(st) + wave * (Cfg::B_CPW * 1024);
#pragma unroll
        for (int t = 0; t < N_COPY; ++t) {
            if (t / PER_PART != part) continue;
            if (t < Cfg::A_CPW)
                __builtin_amdgcn_global_load_lds(PGK_GLB(ga + voff_a[t]), PGK_LDS(la + t * 1024), 16, 0, 0);
            else
                __builtin_amdgcn_global_load_lds(PGK_GLB(gb + voff_b[t - Cfg::A_CPW]),
                                                 PGK_LDS(lb + (t - Cfg::A_CPW) * 1024), 16, 0, 0);
        }
    };
    auto load_tile = [&](int kt, auto st) {
#pragma unroll
        for (int part = 0; part < Cfg::COPY_PARTS; ++part) load_part(kt, st, part);
    };

    // ---- per-lane LDS read offsets
    const int half = lane >> 5;     // which K half of the MFMA operand this lane feeds
    const int l32 = lane & 31;
    // A rows (MFMA "B" operand): row = wave row base + 32 i + l32, logical chunk 2 s + half
    const int a_row_off = (wm * Cfg::WM + l32) * RA;
    int a_koff[NS];                 // per step: row offset + swizzled chunk offset (bytes)
#pragma unroll
    for (int s = 0; s < NS; ++s) a_koff[s] = a_row_off + (((2 * s + half) ^ swz_a<Cfg::A_CPR>(l32)) * 16);
    // B columns (MFMA "A" operand)
    int b_off[TN];
    if constexpr (BF16) {
        const int grp = lane >> 4, pl = lane & 15;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = wn * Cfg::WN + 32 * j + 16 * (grp & 1) + 4 * (pl & 3);
            const int krow = 8 * (grp >> 1) + (pl >> 2);
            const int c = (n >> 3) ^ swz_b<true>(krow);
            b_off[j] = krow * RB + c * 16 + (n & 7) * 2;
        }
    } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = wn * Cfg::WN + 32 * j + l32;
            const int krow = 4 * half;
            const int c = (n >> 2) ^ swz_b<false>(krow);
            b_off[j] = krow * RB + c * 16 + (n & 3) * 4;
        }
    }

    // Operand fragments for one step.  bf16: one step = one MFMA K (16).
    // fp32: one step = 8 K values = four MFMAs per tile pair.
    struct FragBF16 { bf16x8 a[TM]; bf16x8 b[TN]; };
    struct FragF32 { f32x4 a[TM]; float b[4][TN]; };
    using Frag = typename std::conditional<BF16, FragBF16, FragF32>::type;

    auto read_frags = [&](auto st, int s, Frag& f) {
        const unsigned char* as = lds_a(st);
        const unsigned char* bs = lds_b(st);
        if constexpr (BF16) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const unsigned char* q = bs + b_off[j] + (16 * s) * RB;
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4*)PGK_LDS(q));
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4*)PGK_LDS(q + 4 * RB));
                s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                f.b[j] = __builtin_bit_cast(bf16x8, both);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
                f.a[i] = *(const __attribute__((address_space(3))) bf16x8*)PGK_LDS(as + i * 32 * RA + a_koff[s]);
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    f.b[t][j] = *(const __attribute__((address_space(3))) float*)PGK_LDS(bs + b_off[j] + (8 * s + t) * RB);
#pragma unroll
            for (int i = 0; i < TM; ++i)
                f.a[i] = *(const __attribute__((address_space(3))) f32x4*)PGK_LDS(as + i * 32 * RA + a_koff[s]);
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    auto mfma_step = [&](const Frag& f) {
        if constexpr (BF16) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j], f.a[i], acc[i][j], 0, 0, 0);
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f.b[t][j], f.a[i][t], acc[i][j], 0, 0, 0);
        }
    };

    // Wait until at most `allowed` of this wave's direct-to-LDS copy instructions are
    // still in flight (they complete in order), and for its own LDS reads; then meet
    // the other waves.  After the barrier the tile that has just landed is visible to
    // everybody, and everybody has fetched its last operands from the stage that is
    // overwritten next.  The sched_barriers keep the compiler from moving MFMAs or
    // fetches across.
    auto wait_copies_and_sync = [&](auto allowed) {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(decltype(allowed)::value) : "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // copy instructions per wave per tile; tiles kt+2 .. kt+S-1 may stay in flight
    // while tile kt+1 is awaited
    constexpr int STEADY_IN_FLIGHT = (S - 2) * N_COPY;
    static_assert(STEADY_IN_FLIGHT <= 63, "vmcnt is a 6-bit counter");

    Frag frag[2];

    // One K tile out of stage ST.  Operands of step s+1 are fetched while the MFMAs
    // of step s run.  Before the MFMAs of the last step, when a next tile exists:
    // wait for its copy, meet the other waves, fetch its first operands (next
    // stage), and start the copy of tile kt+S into this stage, which nobody reads
    // any more.  That copy is issued in parts: part 0 here, parts 1.. during the
    // first steps of the next tile.  `steady` = every tile up to kt+S exists, so
    // the in-flight count at the wait is the steady-state one; otherwise the wait
    // is for all copies.
    static_assert(Cfg::COPY_PARTS >= 1 && Cfg::COPY_PARTS <= NS, "one copy part per step");
    auto tile_body = [&](int kt, auto st, auto steady_tag, bool has_next, bool has_copy, bool has_prev_copy) {
        constexpr int ST = decltype(st)::value;
        constexpr bool STEADY = decltype(steady_tag)::value != 0;
        using StNext = IC<(ST + 1) % S>;
        using StPrev = IC<(ST + S - 1) % S>;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            bool copy = false;
            if (s + 1 < NS) {
                read_frags(st, s + 1, frag[(s + 1) & 1]);
                if (s + 1 < Cfg::COPY_PARTS && has_prev_copy) {
                    // rest of the copy of tile kt-1+S, started in the previous tile's last step
                    load_part(kt - 1 + S, StPrev{}, s + 1);
                    copy = true;
                }
            } else if (has_next) {
                if constexpr (STEADY) wait_copies_and_sync(IC<STEADY_IN_FLIGHT>{});
                else wait_copies_and_sync(IC<0>{});
                read_frags(StNext{}, 0, frag[0]);
                if (has_copy) {
                    load_part(kt + S, st, 0);
                    copy = true;
                }
            }
            mfma_step(frag[s & 1]);
            // Issue order inside this step: one LDS operand fetch after each MFMA, and
            // the copy instructions of this step evenly spaced over its MFMAs, so the
            // matrix pipe never waits for a burst of fetches.
            constexpr int N_MFMA = BF16 ? TM * TN : 4 * TM * TN;
            constexpr int N_DS = BF16 ? TM + 2 * TN : TM + 4 * TN;
            const bool fetch = (s + 1 < NS) || has_next;
#pragma unroll
            for (int m = 0; m < N_MFMA; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (fetch && m < N_DS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                if (copy && (m * PER_PART) / N_MFMA != ((m + 1) * PER_PART) / N_MFMA)
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
        }
    };

    // prologue: tiles 0 .. S-2 are copied in full; part 0 of tile S-1 follows after
    // the first barrier (its other parts are issued inside tile 0, like every later copy)
    load_tile(0, IC<0>{});
    if constexpr (S > 2) { if (KT > 1) load_tile(1, IC<1>{}); }
    if constexpr (S > 3) { if (KT > 2) load_tile(2, IC<2>{}); }
    if constexpr (S > 4) { if (KT > 3) load_tile(3, IC<3>{}); }
    {
        // tile 0 has landed once at most (tiles issued after it) x N_COPY are in flight
        const int later = (KT - 1 < S - 2) ? KT - 1 : S - 2;
        if (later == 3) wait_copies_and_sync(IC<3 * N_COPY>{});
        else if (later == 2) wait_copies_and_sync(IC<2 * N_COPY>{});
        else if (later == 1) wait_copies_and_sync(IC<N_COPY>{});
        else wait_copies_and_sync(IC<0>{});
    }
    if (KT > S - 1) load_part(S - 1, IC<S - 1>{}, 0);
    read_frags(IC<0>{}, 0, frag[0]);

    int kt = 0;
    // steady state: S tiles per trip, every tile up to kt+2S-1 exists, no conditionals
    for (; kt + 2 * S - 1 < KT; kt += S) {
        tile_body(kt, IC<0>{}, IC<1>{}, true, true, true);
        tile_body(kt + 1, IC<1>{}, IC<1>{}, true, true, true);
        if constexpr (S > 2) tile_body(kt + 2, IC<2>{}, IC<1>{}, true, true, true);
        if constexpr (S > 3) tile_body(kt + 3, IC<3>{}, IC<1>{}, true, true, true);
        if constexpr (S > 4) tile_body(kt + 4, IC<4>{}, IC<1>{}, true, true, true);
    }
    // tail: the remaining (at most 2S-1) tiles, with run-time existence checks and
    // a wait for all copies at each barrier
    auto tail_tile = [&](int t, auto st) {
        if (t < KT) tile_body(t, st, IC<0>{}, t + 1 < KT, t + S < KT, t - 1 + S < KT);
    };
    tail_tile(kt, IC<0>{});
    tail_tile(kt + 1, IC<1 % S>{});
    tail_tile(kt + 2, IC<2 % S>{});
    if constexpr (S > 2) { tail_tile(kt + 3, IC<3 % S>{}); tail_tile(kt + 4, IC<4 % S>{}); }
    if constexpr (S > 3) { tail_tile(kt + 5, IC<5 % S>{}); tail_tile(kt + 6, IC<6 % S>{}); }
    if constexpr (S > 4) { tail_tile(kt + 7, IC<7 % S>{}); tail_tile(kt + 8, IC<8 % S>{}); }

    // ---- epilogue
    const int m_wave = tm * BM + wm * Cfg::WM;
    const int n_wave = tn * BN + wn * Cfg::WN;
    if (out_mode == 1) {
        // split-K pass 1: raw fp32 partial products
        float* w = p.ws + ((size_t)b * p.splits + sp) * (size_t)p.M * (size_t)p.N;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const size_t row_off = (size_t)(m_wave + 32 * i + l32) * (size_t)p.N;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n_wave + 32 * j + 8 * g + 4 * half;
                    f32x4 o = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                    *(f32x4*)(w + row_off + n) = o;
                }
        }
        return;
    }

    float* rs_lds = nullptr;
    if (p.rs_part) {
        __syncthreads();  // every wave is done with the operand tiles; reuse LDS
        rs_lds = (float*)lds_a0 + wn * BM + wm * Cfg::WM;
    }
    const size_t c_base = (size_t)b * p.M * p.N;
    switch (p.act) {
    case ACT_RELU: epilogue_fused<ACT_RELU, BF16, TM, TN>(acc, p, c_base, m_wave, n_wave, lane, rs_lds); break;
    case ACT_GELU_TANH: epilogue_fused<ACT_GELU_TANH, BF16, TM, TN>(acc, p, c_base, m_wave, n_wave, lane, rs_lds); break;
    case ACT_SILU: epilogue_fused<ACT_SILU, BF16, TM, TN>(acc, p, c_base, m_wave, n_wave, lane, rs_lds); break;
    default: epilogue_fused<ACT_NONE, BF16, TM, TN>(acc, p, c_base, m_wave, n_wave, lane, rs_lds); break;
    }
    if (p.rs_part) {
        __syncthreads();
        if (tid < BM) {
            const float* r = (const float*)lds_a0 + tid;
            float s = r[0];
#pragma unroll
            for (int w = 1; w < Cfg::WGN; ++w) s += r[w * BM];
            p.rs_part[((size_t)b * p.tiles_n + tn) * (size_t)p.M + (size_t)tm * BM + tid] = s;
        }
    }
}

// Shipping configurations: <bf16, BM, BN, BK, wave rows, wave cols, copy parts, stages, waves/SIMD>.
// bf16: 256x256x64 tile, eight waves of 64x128 (two per SIMD, so one wave's operand
// fetches and barrier waits overlap the other's MFMAs), 128 KiB of LDS.
// fp32: 128x128x32 tile, four waves of 64x64, 64 KiB of LDS, two workgroups per CU.
using CfgBF16 = MfmaCfg<true, 256, 256, 64, 4, 2, 2, 2, 2>;
using CfgF32 = MfmaCfg<false, 128, 128, 32, 2, 2, 1, 2, 1>;

TileShape mfma_tile_shape(int dtype)
{
    if (dtype == DT_BF16) return {CfgBF16::BM, CfgBF16::BN, CfgBF16::BK};
    return {CfgF32::BM, CfgF32::BN, CfgF32::BK};
}

template <typename Cfg>
static hipError_t launch_cfg(const GemmArgs& a, int out_mode, hipStream_t s)
{
    const long long wgs = (long long)a.tiles_m * a.tiles_n * a.batch * a.splits;
    if (wgs <= 0 || wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gemm_mfma_kernel<Cfg>, dim3((unsigned int)wgs), dim3(Cfg::NT), 0, s, a, out_mode);
    return hipGetLastError();
}

hipError_t launch_gemm_mfma(const GemmArgs& a, int dtype, int out_mode, hipStream_t s)
{
    if (dtype == DT_BF16) return launch_cfg<CfgBF16>(a, out_mode, s);
    return launch_cfg<CfgF32>(a, out_mode, s);
}

}  // namespace pgk
