"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element on the same seeded inputs.

Error bar: max |g - r| / max(|r|, RMS(r)) <= 1e-4 for fp32 and <= 2e-2 for bf16
inputs with fp32 accumulation; integer-valued inputs with the identity activation
must match the oracle exactly (every fp32 summation order is exact there).
"""
import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen
from util import TOL, abs_inputs, c_to_numpy, rel_err, sample_rows, strict_rel_err, to_device

pytestmark = pytest.mark.gpu

NONE, RELU, GELU, SILU = gen.ACT_NONE, gen.ACT_RELU, gen.ACT_GELU_TANH, gen.ACT_SILU
F32, BF16 = gen.F32, gen.BF16


@pytest.fixture(scope="module")
def pgk():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2511_06345_amd import binding
    binding.load_library()          # fails loudly when libpgk.so is missing: there is no fallback
    return binding


def run_fused(pgk, A, B, bias, act, dtype, rowsum=True):
    import torch
    dA, dB = to_device(A, dtype), to_device(B, dtype)
    dbias = torch.from_numpy(bias).cuda() if bias is not None else None
    C, rs = pgk.gemm_fused(dA, dB, dbias, act, rowsum=rowsum)
    torch.cuda.synchronize()
    return c_to_numpy(C, dtype), (rs.cpu().numpy().astype(np.float64) if rs is not None else None)


def run_splitk(pgk, A, B, bias, act, dtype, splits=0, rowsum=True):
    import torch
    dA, dB = to_device(A, dtype), to_device(B, dtype)
    dbias = torch.from_numpy(bias).cuda() if bias is not None else None
    C, rs = pgk.gemm_splitk(dA, dB, dbias, act, splits=splits, rowsum=rowsum)
    torch.cuda.synchronize()
    return c_to_numpy(C, dtype), (rs.cpu().numpy().astype(np.float64) if rs is not None else None)


def random_case(dtype, M, N, K, batch, seed, bias_std=0.5):
    rng_seed = 1000 + seed
    A = gen.uniform(gen.tensor_seed(90, 1, rng_seed), batch * M * K, -1.0, 1.0).reshape(batch, M, K)
    B = gen.uniform(gen.tensor_seed(90, 2, rng_seed), batch * K * N, -1.0, 1.0).reshape(batch, K, N)
    bias = gen.normal(gen.tensor_seed(90, 3, rng_seed), N, bias_std)
    if dtype == BF16:
        A, B = gen.f32_to_bf16_bits(A), gen.f32_to_bf16_bits(B)
    return A, B, bias


def check(got_c, got_rs, ref_c, ref_rs, dtype, what):
    e = rel_err(got_c, ref_c)
    assert e <= TOL[dtype], f"{what}: C error {e:.3e}"
    if ref_rs is not None and got_rs is not None:
        e = rel_err(got_rs, ref_rs)
        assert e <= TOL[dtype], f"{what}: rowsum error {e:.3e}"


# shapes: tiny and ragged (outputs below 16 x 16 and problems too small to copy operands for run on
# the bounds-checked kernel, the others on the matrix cores in place or from padded copies), exact
# tile multiples with several K-tile counts, and mixes with a ragged tail in each dimension
GUARDED_SHAPES = [(1, 1, 1, 1), (5, 7, 33, 2), (65, 63, 17, 1), (130, 70, 100, 3), (64, 64, 16, 1), (2, 300, 5, 1),
                  (15, 15, 1000, 2), (9, 14, 513, 3), (1, 15, 1023, 1), (33, 31, 255, 1), (60, 61, 63, 1)]
# K a whole number of K tiles, M and N ragged: matrix-core kernels with edge tiles
F32_EDGE_SHAPES = [(100, 36, 64, 2), (129, 132, 96, 1), (300, 260, 32, 1), (17, 500, 128, 1), (250, 16, 64, 3)]
BF16_EDGE_SHAPES = [(100, 40, 64, 2), (257, 264, 128, 1), (300, 520, 64, 1), (17, 1000, 192, 1), (700, 16, 64, 2)]
# K a multiple of the 16-byte chunk only (4 fp32 / 8 bf16 elements): the last K tile is
# partial, with one to sixteen full tiles before it
F32_KTAIL_SHAPES = [(128, 128, 36, 1), (100, 36, 4, 2), (129, 132, 100, 1), (256, 128, 60, 2), (64, 64, 200, 3), (70, 200, 524, 1)]
BF16_KTAIL_SHAPES = [(256, 256, 72, 1), (100, 40, 8, 2), (257, 264, 200, 1), (300, 520, 120, 2), (128, 128, 456, 2), (256, 128, 520, 1), (130, 72, 1032, 1)]
F32_TILE_SHAPES = [(128, 128, 32, 1), (128, 128, 64, 1), (256, 128, 96, 1), (128, 384, 160, 2), (384, 256, 224, 1)]
BF16_TILE_SHAPES = [(256, 256, 64, 1), (256, 256, 128, 1), (256, 512, 192, 1), (512, 256, 320, 2), (256, 256, 448, 1)]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("shape", GUARDED_SHAPES)
@pytest.mark.parametrize("act", [NONE, RELU, GELU, SILU])
def test_small_and_ragged_shapes(pgk, oracle, dtype, shape, act):
    M, N, K, batch = shape
    A, B, bias = random_case(dtype, M, N, K, batch, seed=M + N + K)
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, act)
    got_c, got_rs = run_fused(pgk, A, B, bias, act, dtype)
    check(got_c, got_rs, ref_c, ref_rs, dtype, f"guarded {shape} act {act}")


@pytest.mark.parametrize("dtype,shapes", [(F32, F32_TILE_SHAPES + F32_EDGE_SHAPES + F32_KTAIL_SHAPES),
                                          (BF16, BF16_TILE_SHAPES + BF16_EDGE_SHAPES + BF16_KTAIL_SHAPES)])
@pytest.mark.parametrize("act", [NONE, RELU, GELU, SILU])
def test_tile_multiple_shapes(pgk, oracle, dtype, shapes, act):
    for shape in shapes:
        M, N, K, batch = shape
        A, B, bias = random_case(dtype, M, N, K, batch, seed=M + 3 * N + 7 * K)
        ref_c, ref_rs = oracle.gemm_fused(A, B, bias, act)
        got_c, got_rs = run_fused(pgk, A, B, bias, act, dtype)
        check(got_c, got_rs, ref_c, ref_rs, dtype, f"mfma {shape} act {act}")
        # no bias, no row sum
        ref_c, _ = oracle.gemm_fused(A, B, None, act, want_rowsum=False)
        got_c, got_rs = run_fused(pgk, A, B, None, act, dtype, rowsum=False)
        assert got_rs is None
        check(got_c, None, ref_c, None, dtype, f"mfma {shape} act {act} no bias")


@pytest.mark.parametrize("dtype,shapes", [(F32, F32_TILE_SHAPES + F32_EDGE_SHAPES + F32_KTAIL_SHAPES + GUARDED_SHAPES),
                                          (BF16, BF16_TILE_SHAPES + BF16_EDGE_SHAPES + BF16_KTAIL_SHAPES + GUARDED_SHAPES)])
def test_integer_inputs_are_exact(pgk, oracle, dtype, shapes):
    """Entries in {-2..2}, identity activation: bit-exact against the oracle, for every
    K-tile count (catches stage / double-buffer hazards and index slips)."""
    for shape in shapes:
        M, N, K, batch = shape
        A, B = gen.make_int_inputs(dtype, M, N, K, batch, seed=11 * M + K)
        ref_c, ref_rs = oracle.gemm_fused(A, B, None, NONE)
        got_c, got_rs = run_fused(pgk, A, B, None, NONE, dtype)
        if dtype == BF16:   # C is stored as bf16: compare against the RNE-rounded exact value
            ref_c = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref_c.astype(np.float32))).astype(np.float64)
        assert np.array_equal(got_c, ref_c), f"fused {shape}"
        assert np.array_equal(got_rs, ref_rs), f"fused rowsum {shape}"
        for splits in (0, 1, 2, 3):
            if splits > K:
                continue
            got_c, got_rs = run_splitk(pgk, A, B, None, NONE, dtype, splits=splits)
            assert np.array_equal(got_c, ref_c), f"splitk {shape} splits {splits}"
            assert np.array_equal(got_rs, ref_rs), f"splitk rowsum {shape} splits {splits}"


# The library picks its small tile (64x64 fp32, 128x128 bf16) when the large-tile grid
# would have fewer than 192 workgroups, so the shapes above run on the small tiles.  These
# have enough batch entries to get the large tiles (128x128 fp32, 256x256 bf16), with
# one to seven K tiles and ragged edges.
LARGE_TILE_SHAPES = {F32: [(128, 128, 32, 192), (256, 128, 96, 100), (300, 260, 64, 40), (129, 140, 224, 70),
                           (128, 128, 36, 192), (300, 260, 100, 40), (129, 140, 300, 70)],
                     BF16: [(256, 256, 64, 192), (512, 256, 192, 100), (300, 520, 128, 40), (257, 264, 448, 50),
                            (256, 256, 72, 192), (300, 520, 200, 40), (257, 264, 520, 50), (256, 256, 1032, 48),
                            # last tile column / row at most half full: the 256x128 and 128x256 tiles
                            (512, 128, 192, 100), (300, 100, 200, 100), (256, 128, 1032, 192), (1024, 72, 64, 50),
                            (128, 512, 192, 100), (100, 300, 520, 100), (128, 256, 72, 192), (72, 1024, 448, 50)]}


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_large_tiles_with_many_batch_entries(pgk, oracle, dtype):
    for shape in LARGE_TILE_SHAPES[dtype]:
        M, N, K, batch = shape
        A, B = gen.make_int_inputs(dtype, M, N, K, batch, seed=3 * M + K)
        ref_c, ref_rs = oracle.gemm_fused(A, B, None, NONE)
        got_c, got_rs = run_fused(pgk, A, B, None, NONE, dtype)
        if dtype == BF16:
            ref_c = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref_c.astype(np.float32))).astype(np.float64)
        assert np.array_equal(got_c, ref_c), f"large tile {shape}"
        assert np.array_equal(got_rs, ref_rs), f"large tile rowsum {shape}"
        got_c, got_rs = run_splitk(pgk, A, B, None, NONE, dtype, splits=2)
        assert np.array_equal(got_c, ref_c) and np.array_equal(got_rs, ref_rs), f"large tile split-K {shape}"
        A, B, bias = random_case(dtype, M, N, K, batch, seed=M + K)
        ref_c, ref_rs = oracle.gemm_fused(A, B, bias, GELU)
        got_c, got_rs = run_fused(pgk, A, B, bias, GELU, dtype)
        check(got_c, got_rs, ref_c, ref_rs, dtype, f"large tile {shape} GELU")


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("act", [NONE, SILU])
def test_splitk_matches_oracle_and_is_deterministic(pgk, oracle, dtype, act):
    # the last two are skinny: the second pass cuts their columns into segments and the row
    # sums are combined from per-segment partials
    shapes = [(128, 128, 1024, 3), (256, 256, 2048, 2), (100, 36, 1000, 2), (20, 2056, 512, 1), (16, 4096, 256, 2)]
    for shape in shapes:
        M, N, K, batch = shape
        A, B, bias = random_case(dtype, M, N, K, batch, seed=5 * M + K)
        ref_c, ref_rs = oracle.gemm_fused(A, B, bias, act)
        for splits in (0, 4, 7):
            got_c, got_rs = run_splitk(pgk, A, B, bias, act, dtype, splits=splits)
            check(got_c, got_rs, ref_c, ref_rs, dtype, f"splitk {shape} splits {splits}")
            again_c, again_rs = run_splitk(pgk, A, B, bias, act, dtype, splits=splits)
            assert np.array_equal(got_c, again_c) and np.array_equal(got_rs, again_rs)
        fused_c, fused_rs = run_fused(pgk, A, B, bias, act, dtype)
        check(fused_c, fused_rs, ref_c, ref_rs, dtype, f"fused {shape}")


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("batch", [2, 48])
def test_k_tail_ignores_what_follows_a_row(pgk, oracle, dtype, batch):
    """K not a multiple of the K tile: the columns of the last tile that do not exist lie,
    in memory, over the start of the next row of A and over the next batch entry of B.
    NaNs planted there must not reach the rows / batch entries before them."""
    M, N, K = 260, 264, 200 if dtype == BF16 else 100
    A, B, bias = random_case(dtype, M, N, K, batch, seed=77)
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, NONE)
    nan = np.uint16(0x7FC0) if dtype == BF16 else np.float32(np.nan)
    bad_row, bad_batch = 131, batch - 1
    A2, B2 = A.copy(), B.copy()
    A2[:, bad_row, :16] = nan           # what the tail columns of row 130 run into
    B2[bad_batch, :16, :] = nan         # what the tail rows of B of the batch entry before run into
    got_c, got_rs = run_fused(pgk, A2, B2, bias, NONE, dtype)
    keep = np.ones((batch, M), dtype=bool)
    keep[:, bad_row] = False
    keep[bad_batch, :] = False
    assert np.all(np.isfinite(got_c[keep])) and np.all(np.isfinite(got_rs[keep]))
    assert np.all(np.isnan(got_c[~keep]))
    for b in range(batch - 1):
        check(got_c[b][keep[b]], got_rs[b][keep[b]], ref_c[b][keep[b]], ref_rs[b][keep[b]], dtype, f"batch {b}")


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_skinny_splitk_is_exact_on_integers(pgk, oracle, dtype):
    for shape in [(16, 4096, 512, 1), (40, 1288, 256, 3), (7, 3000, 128, 2)]:
        M, N, K, batch = shape
        A, B = gen.make_int_inputs(dtype, M, N, K, batch, seed=M + N)
        ref_c, ref_rs = oracle.gemm_fused(A, B, None, NONE)
        if dtype == BF16:
            ref_c = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref_c.astype(np.float32))).astype(np.float64)
        for splits in (0, 2, 5):
            got_c, got_rs = run_splitk(pgk, A, B, None, NONE, dtype, splits=splits)
            assert np.array_equal(got_c, ref_c) and np.array_equal(got_rs, ref_rs), f"{shape} splits {splits}"


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("which", ["A", "B", "C", "bias", "workspace"])
def test_pointers_off_the_16_byte_grid(pgk, oracle, dtype, which):
    """A tile-friendly shape with one pointer a single element past a 16-byte boundary: a
    misaligned operand is copied first, C and the bias are used where they are (their rows may
    start on any element), all with the same result; a misaligned workspace is refused."""
    import torch
    M, N, K, batch = 128, 256, 192, 2
    A, B, bias = random_case(dtype, M, N, K, batch, seed=41)
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, SILU)
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32

    def shifted(t):
        flat = torch.empty(t.numel() + 1, dtype=t.dtype, device="cuda")
        v = flat[1:].view(t.shape)
        v.copy_(t)
        assert v.data_ptr() % 16 != 0 and v.is_contiguous()
        return v

    dA, dB, dbias = to_device(A, dtype), to_device(B, dtype), torch.from_numpy(bias).cuda()
    C = torch.empty((batch, M, N), dtype=tdt, device="cuda")
    if which == "A":
        dA = shifted(dA)
    elif which == "B":
        dB = shifted(dB)
    elif which == "C":
        C = shifted(C)
    elif which == "bias":
        dbias = shifted(dbias)
    if which == "workspace":
        need = pgk.splitk_workspace_bytes(M, N, K, batch, dtype, 2)
        ws = torch.empty(need + 16, dtype=torch.uint8, device="cuda")[4:]
        with pytest.raises(pgk.PgkError) as ei:      # the workspace is the caller's: it must be aligned
            pgk.gemm_splitk(dA, dB, dbias, SILU, splits=2, out=C, workspace=ws)
        assert ei.value.status == -3
        return
    C, rs = pgk.gemm_fused(dA, dB, dbias, SILU, out=C)
    torch.cuda.synchronize()
    check(c_to_numpy(C, dtype), rs.cpu().numpy().astype(np.float64), ref_c, ref_rs, dtype, f"misaligned {which}")
    C2, rs2 = pgk.gemm_splitk(dA, dB, dbias, SILU, splits=3, out=torch.empty_like(C))
    torch.cuda.synchronize()
    check(c_to_numpy(C2, dtype), rs2.cpu().numpy().astype(np.float64), ref_c, ref_rs, dtype, f"misaligned {which}, split")


# Latency-bound fp32 problems: 32 x 32 tiles whose four waves split K (pgk_gemm_tiny.hip).  Ragged M
# and N (multiples of 4), K with a partial last step, fewer K steps than waves, several batch entries.
TINY_SHAPES = [(256, 256, 256, 1), (40, 36, 64, 1), (100, 200, 992, 2), (512, 512, 68, 1), (257, 260, 500, 1),
               (33, 64, 96, 5), (129, 36, 128, 3)]


@pytest.mark.parametrize("act", [NONE, RELU, GELU, SILU])
def test_k_splitting_tile_for_latency_bound_problems(pgk, oracle, act):
    for shape in TINY_SHAPES:
        M, N, K, batch = shape
        assert pgk.gemm_plan(M, N, K, batch, F32)["tile"] == (32, 32, 32), shape
        A, B, bias = random_case(F32, M, N, K, batch, seed=M + 5 * N + K)
        ref_c, ref_rs = oracle.gemm_fused(A, B, bias, act)
        got_c, got_rs = run_fused(pgk, A, B, bias, act, F32)
        check(got_c, got_rs, ref_c, ref_rs, F32, f"tiny {shape} act {act}")
        again_c, again_rs = run_fused(pgk, A, B, bias, act, F32)
        assert np.array_equal(got_c, again_c) and np.array_equal(got_rs, again_rs), f"tiny {shape}: run-to-run difference"
        if act == NONE:
            Ai, Bi = gen.make_int_inputs(F32, M, N, K, batch, seed=7 * M + K)
            ref_c, ref_rs = oracle.gemm_fused(Ai, Bi, None, NONE)
            got_c, got_rs = run_fused(pgk, Ai, Bi, None, NONE, F32)
            assert np.array_equal(got_c, ref_c) and np.array_equal(got_rs, ref_rs), f"tiny {shape}: integers"
            got_c, got_rs = run_fused(pgk, Ai, Bi, None, NONE, F32, rowsum=False)
            assert got_rs is None and np.array_equal(got_c, ref_c)


@pytest.mark.parametrize("dtype,shape", [(BF16, (520, 776, 200)), (BF16, (256, 256, 64)), (F32, (260, 392, 100)),
                                         (F32, (128, 128, 32))])
@pytest.mark.parametrize("act", [NONE, GELU])
def test_measurement_instance_computes_what_the_kernel_computes(pgk, oracle, dtype, shape, act):
    """pgk_probe_gemm_phases: the large-tile kernel of either type with phase stamps.  Its C and its
    per-tile-column partial row sums meet the oracle to the same bar as the fused call, and every
    workgroup leaves six stamps in time order."""
    import torch
    M, N, K = shape
    bm, bn = (256, 256) if dtype == BF16 else (128, 128)
    A, B, bias = random_case(dtype, M, N, K, 1, seed=M + N + K)
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, act)
    dA, dB = to_device(A, dtype), to_device(B, dtype)
    tiles_n, wgs = -(-N // bn), -(-M // bm) * -(-N // bn)
    C = torch.empty((1, M, N), dtype=dA.dtype, device="cuda")
    part = torch.full((tiles_n, M), float("nan"), dtype=torch.float32, device="cuda")
    stamps = torch.zeros((wgs, pgk.STAMP_WORDS), dtype=torch.int64, device="cuda")
    assert pgk.probe_gemm_phases(dA, dB, torch.from_numpy(bias).cuda(), act, C, stamps, rowsum_partials=part) == wgs
    torch.cuda.synchronize()
    got_rs = part.cpu().numpy().astype(np.float64).sum(axis=0)[None, :]
    check(c_to_numpy(C, dtype), got_rs, ref_c, ref_rs, dtype, f"timed instance {shape} act {act}")
    st = stamps.cpu().numpy()
    cycles, ticks = st[:, 0:12:2], st[:, 1:12:2]
    assert np.all(np.diff(cycles, axis=1) > 0) and np.all(np.diff(ticks, axis=1) >= 0)
    # too little room for the stamps: refused before any launch
    with pytest.raises(pgk.PgkError):
        pgk.probe_gemm_phases(dA, dB, None, act, C, stamps.reshape(-1)[:wgs * pgk.STAMP_WORDS - 1].clone())


def test_fed_matrix_instruction_probe_runs_and_reports_its_clock(pgk):
    """pgk_probe_mfma_fed (a measurement aid): every form finishes, reports cycles and ticks of a
    plausible shader clock, and leaves its source untouched."""
    import torch
    clock = torch.zeros(4, dtype=torch.int64, device="cuda")
    src = (torch.randn((8 << 20) // 2, device="cuda") * 0.01).to(torch.bfloat16)       # 8 MiB: 128 pieces
    before = src.clone()
    for kw in ({}, {"src": src, "resident_bytes": 1 << 20}, {"src": src, "resident_bytes": 1 << 20, "stream_every": 3}):
        clock.zero_()
        flops = pgk.probe_mfma_fed(64, clock, **kw)
        torch.cuda.synchronize()
        assert flops == 2.0 * 32 * 32 * 16 * 32 * 64 * 8 * 256
        cycles, ticks, alive = (int(v) for v in clock[:3].cpu())
        assert alive == 0 and ticks > 0 and 0.4 <= cycles / ticks * 0.1 <= 2.6, (cycles, ticks)
    assert torch.equal(src, before)
    with pytest.raises(pgk.PgkError):
        pgk.probe_mfma_fed(63, clock)


def test_identity_operand_passes_b_through(pgk, oracle):
    # A = I: C = act(B + bias) -- exercises operand roles (a transposed B would fail)
    n = 256
    B = gen.normal(1234, n * n, 1.0).reshape(1, n, n)
    bias = gen.normal(1235, n, 1.0)
    A = np.eye(n, dtype=np.float32).reshape(1, n, n)
    for dtype in (F32, BF16):
        a, b = (gen.f32_to_bf16_bits(A), gen.f32_to_bf16_bits(B)) if dtype == BF16 else (A, B)
        ref_c, ref_rs = oracle.gemm_fused(a, b, bias, RELU)
        got_c, got_rs = run_fused(pgk, a, b, bias, RELU, dtype)
        check(got_c, got_rs, ref_c, ref_rs, dtype, "identity operand")


def test_fused_is_deterministic(pgk):
    for dtype, shape in ((F32, (256, 384, 96, 2)), (BF16, (512, 512, 128, 1)), (F32, (70, 130, 33, 2))):
        M, N, K, batch = shape
        A, B, bias = random_case(dtype, M, N, K, batch, seed=3)
        c1, r1 = run_fused(pgk, A, B, bias, GELU, dtype)
        c2, r2 = run_fused(pgk, A, B, bias, GELU, dtype)
        assert np.array_equal(c1, c2) and np.array_equal(r1, r2)


def test_error_codes_on_device(pgk):
    import torch
    a = torch.zeros(1, 8, 8, device="cuda")
    with pytest.raises(pgk.PgkError) as ei:
        pgk.gemm_splitk(a, a, None, NONE, splits=9)              # splits > K
    assert ei.value.status == -1
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(pgk.PgkError) as ei:
        pgk.gemm_splitk(a, a, None, NONE, splits=1, workspace=small)
    assert ei.value.status == -3


# ------------------------------------------------------------------ the five workloads
def _workload_case(pgk, oracle, name):
    """A workload at its full size, in the configuration bench.py times, against the oracle on
    EVERY element of C and of the row sums; two runs must agree bit for bit.  Prints, unjudged, the
    strict relative error over the entries of at least RMS size and the error relative to the
    a-priori scale sum_k |a||b| + |bias| (the running-error bound's denominator)."""
    import torch
    w = gen.WORKLOADS[name]
    A, B, bias = gen.make_inputs(w)
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, w.act, want_rowsum=w.rowsum)
    dA, dB = to_device(A, w.dtype), to_device(B, w.dtype)
    dbias = torch.from_numpy(bias).cuda() if bias is not None else None
    fn = pgk.gemm_splitk if w.call == "splitk" else pgk.gemm_fused
    C, rs = fn(dA, dB, dbias, w.act, rowsum=w.rowsum)
    torch.cuda.synchronize()
    C2, rs2 = fn(dA, dB, dbias, w.act, rowsum=w.rowsum)
    torch.cuda.synchronize()
    assert torch.equal(C.view(torch.int16 if w.dtype == BF16 else torch.int32),
                       C2.view(torch.int16 if w.dtype == BF16 else torch.int32)), "run-to-run difference"
    if rs is not None:
        assert torch.equal(rs, rs2)
    del C2, rs2
    got_c = c_to_numpy(C, w.dtype)
    got_rs = rs.cpu().numpy().astype(np.float64) if rs is not None else None
    check(got_c, got_rs, ref_c, ref_rs, w.dtype, f"workload {name}")
    # unjudged figures
    aa, ab, abias = abs_inputs(A, B, bias, w.dtype)
    # (the scale costs a second pass of the oracle: on the largest workload, 512 seeded rows of it)
    rows = sample_rows(w.M, 256, 128, seed=w.index) if w.flops > 5e11 else np.arange(w.M, dtype=np.int64)
    scale, _ = oracle.gemm_fused(aa, ab, abias, NONE, rows=rows, want_rowsum=False)
    higham = float(np.max(np.abs(got_c[:, rows] - ref_c[:, rows]) / np.maximum(scale, np.finfo(np.float64).tiny)))
    print(f"\n[{name}] all {got_c.size} elements: judged error {rel_err(got_c, ref_c):.3e} (bar {TOL[w.dtype]:.0e}); "
          f"strict relative error over |ref| >= RMS {strict_rel_err(got_c, ref_c):.3e}; "
          f"max |g - r| / (sum_k |a||b| + |bias|) {higham:.3e}; max absolute error {np.max(np.abs(got_c - ref_c)):.3e}"
          + (f"; row sums judged {rel_err(got_rs, ref_rs):.3e}, strict {strict_rel_err(got_rs, ref_rs):.3e}"
             if got_rs is not None else ""))
    return rel_err(got_c, ref_c)


def test_workload_c1_full(pgk, oracle):
    _workload_case(pgk, oracle, "c1")


def test_workload_c2_full(pgk, oracle):
    _workload_case(pgk, oracle, "c2")


def test_workload_c3_full(pgk, oracle):
    _workload_case(pgk, oracle, "c3")


def test_workload_c4_full(pgk, oracle):
    _workload_case(pgk, oracle, "c4")


def test_workload_c5_full(pgk, oracle):
    _workload_case(pgk, oracle, "c5")


@pytest.mark.parametrize("shape", [(65536, 128, 1024), (128, 65536, 1024)])
def test_skinny_full_size_sampled_rows(pgk, oracle, shape):
    """One dimension of 128: the half-width / half-height bf16 tiles at full size (256 workgroups)."""
    import torch
    M, N, K = shape
    A = gen.f32_to_bf16_bits(gen.normal(gen.tensor_seed(94, 1, M), M * K, 1.0).reshape(1, M, K))
    B = gen.f32_to_bf16_bits(gen.normal(gen.tensor_seed(94, 2, M), K * N, 1.0 / 32).reshape(1, K, N))
    bias = gen.normal(gen.tensor_seed(94, 3, M), N, 0.5)
    rows = sample_rows(M, 128, 32, seed=3)
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, GELU, rows=rows)
    C, rs = pgk.gemm_fused(to_device(A, BF16), to_device(B, BF16), torch.from_numpy(bias).cuda(), GELU)
    torch.cuda.synchronize()
    drows = torch.from_numpy(rows).cuda()
    check(c_to_numpy(C[:, drows], BF16), rs[:, drows].cpu().numpy().astype(np.float64), ref_c, ref_rs, BF16, f"skinny {shape}")


@pytest.mark.parametrize("dtype,K", [(F32, 256), (BF16, 512)])
def test_output_larger_than_4_gib_of_offsets(pgk, oracle, dtype, K):
    """C of 32768 x 32768: 2^30 elements, 4 GiB as fp32 -- element and byte offsets of the last
    rows do not fit 32 bits.  Sampled rows (first, last, tile boundaries, random), C and row sums."""
    import torch
    M = N = 32768
    A = gen.uniform(gen.tensor_seed(97, 1, K), M * K, -1.0, 1.0).reshape(1, M, K)
    B = gen.uniform(gen.tensor_seed(97, 2, K), K * N, -1.0, 1.0).reshape(1, K, N)
    bias = gen.normal(gen.tensor_seed(97, 3, K), N, 0.5)
    if dtype == BF16:
        A, B = gen.f32_to_bf16_bits(A), gen.f32_to_bf16_bits(B)
    rows = sample_rows(M, 256, 24, seed=K)
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, RELU, rows=rows)
    C, rs = pgk.gemm_fused(to_device(A, dtype), to_device(B, dtype), torch.from_numpy(bias).cuda(), RELU)
    torch.cuda.synchronize()
    drows = torch.from_numpy(rows).cuda()
    check(c_to_numpy(C[:, drows], dtype), rs[:, drows].cpu().numpy().astype(np.float64), ref_c, ref_rs, dtype,
          f"large output dtype {dtype}")
    del C, rs
    torch.cuda.empty_cache()


@pytest.mark.parametrize("N", [64, 512])      # small tiles / large tiles
def test_operand_larger_than_4_gib(pgk, oracle, N):
    """A of 66560 x 32776 bf16 (4.36 GB; a seeded block of 1024 rows repeated): byte offsets of
    its last rows exceed 32 bits, K has a partial last tile, and the copies of that tile for the
    last rows run up to the end of the array.  Sampled rows against the oracle."""
    import torch
    rows_block, reps, K = 1024, 65, 32776
    M = rows_block * reps
    block = gen.f32_to_bf16_bits(gen.uniform(gen.tensor_seed(98, 1, 0), rows_block * K, -1.0, 1.0).reshape(rows_block, K))
    B = gen.f32_to_bf16_bits(gen.uniform(gen.tensor_seed(98, 2, 0), K * N, -1.0, 1.0).reshape(1, K, N))
    dblock = to_device(block, BF16)
    dA = dblock.repeat(reps, 1).reshape(1, M, K)
    assert dA.numel() * 2 > (1 << 32)
    C, rs = pgk.gemm_fused(dA, to_device(B, BF16), None, NONE)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([sample_rows(M, 256, 16, seed=1), np.arange(M - 8, M)]))
    ref_c, ref_rs = oracle.gemm_fused(block[rows % rows_block][None], B, None, NONE)
    drows = torch.from_numpy(rows).cuda()
    check(c_to_numpy(C[:, drows], BF16), rs[:, drows].cpu().numpy().astype(np.float64), ref_c, ref_rs, BF16, "large A")
    # equal rows of A give equal rows of C, wherever they lie
    assert torch.equal(C[0, :rows_block].view(torch.int16), C[0, M - rows_block:].view(torch.int16))
    del dA, C
    torch.cuda.empty_cache()


def test_workload_c3_without_bias_or_activation(pgk, oracle):
    """The large bf16 workload is bias dominated; check the bare product too."""
    import torch
    w = gen.WORKLOADS["c3"]
    A, B, _ = gen.make_inputs(w, shape=(1024, 1024, 8192, 1))
    rows = sample_rows(1024, 256, 32, seed=9)
    ref_c, _ = oracle.gemm_fused(A, B, None, NONE, rows=rows, want_rowsum=False)
    C, _ = pgk.gemm_fused(to_device(A, BF16), to_device(B, BF16), None, NONE, rowsum=False)
    torch.cuda.synchronize()
    got = c_to_numpy(C[:, torch.from_numpy(rows).cuda()], BF16)
    check(got, None, ref_c, None, BF16, "c3 bare product")
