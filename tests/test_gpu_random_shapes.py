"""GPU parity on seeded random shapes: every call (fused, split, either layout of B) on sizes drawn
so that each kernel path is reached -- bounds-checked kernel, small / large / half tiles with
ragged edges and a partial last K tile, the automatic split -- against the CPU oracle.

Integer-valued cases (entries in {-2..2}, identity) must match exactly; the others within
1e-4 (fp32) / 2e-2 (bf16) on max |g - r| / max(|r|, RMS(r)).
"""
import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen
from util import TOL, c_to_numpy, rel_err, to_device

pytestmark = pytest.mark.gpu

F32, BF16 = gen.F32, gen.BF16
ACTS = [gen.ACT_NONE, gen.ACT_RELU, gen.ACT_GELU_TANH, gen.ACT_SILU]
CALLS = ["fused", "fused_bt", "splitk", "splitk_bt"]


@pytest.fixture(scope="module")
def pgk():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2511_06345_amd import binding
    binding.load_library()
    return binding


def draw_cases(seed, count):
    """(dtype, M, N, K, batch) per size class; K and N mostly on the 16-byte grid, sometimes off
    it (the matrix-core kernels on zero-padded copies, or the bounds-checked kernel when small)."""
    rng = np.random.default_rng(seed)
    cases = []
    for n in range(count):
        dtype = BF16 if rng.integers(2) else F32
        step = 8 if dtype == BF16 else 4
        big = 256 if dtype == BF16 else 128
        kind = ["any", "grid", "large", "tall", "wide", "longk"][n % 6]
        on_grid = lambda v: max(step, int(v) // step * step)
        if kind == "any":      # every other one too small for the operands to be copied: bounds-checked kernel
            hi = 60 if (n // 6) % 2 else 300
            M, N, K, batch = int(rng.integers(1, hi)), int(rng.integers(1, hi)), int(rng.integers(1, hi)), int(rng.integers(1, 4))
        elif kind == "grid":
            M, N, K, batch = int(rng.integers(16, 700)), on_grid(rng.integers(16, 700)), on_grid(rng.integers(step, 900)), int(rng.integers(1, 4))
        elif kind == "large":      # enough batch entries for the large-tile grid to reach 192 workgroups
            M, N, K = int(rng.integers(big, 3 * big)), on_grid(rng.integers(big, 3 * big)), on_grid(rng.integers(step, 700))
            batch = -(-192 // (-(-M // big) * -(-N // big)))
        elif kind == "tall":       # last tile column at most half full
            M, N, K = int(rng.integers(big, 3 * big)), on_grid(rng.integers(big // 4 + step, big // 2 + 1)), on_grid(rng.integers(step, 500))
            batch = -(-192 // -(-M // big))
        elif kind == "wide":
            M, N, K = int(rng.integers(big // 4 + 1, big // 2 + 1)), on_grid(rng.integers(big, 3 * big)), on_grid(rng.integers(step, 500))
            batch = -(-192 // -(-N // big))
        else:                      # few tiles, long K: the fused call splits by itself
            M, N, K, batch = int(rng.integers(16, 200)), on_grid(rng.integers(16, 400)), on_grid(rng.integers(2048, 6000)), int(rng.integers(1, 3))
        cases.append((dtype, M, N, K, batch))
    return cases


CASES = draw_cases(20251127, 48)


def run(pgk, call, A, B, bias, act, dtype, rowsum, splits):
    import torch
    bt = call.endswith("_bt")
    if bt:
        B = np.ascontiguousarray(np.swapaxes(B, 1, 2))
    dA, dB = to_device(A, dtype), to_device(B, dtype)
    dbias = torch.from_numpy(bias).cuda() if bias is not None else None
    if call.startswith("fused"):
        C, rs = pgk.gemm_fused(dA, dB, dbias, act, rowsum=rowsum, b_transposed=bt)
    else:
        C, rs = pgk.gemm_splitk(dA, dB, dbias, act, splits=splits, rowsum=rowsum, b_transposed=bt)
    torch.cuda.synchronize()
    return c_to_numpy(C, dtype), (rs.cpu().numpy().astype(np.float64) if rs is not None else None)


@pytest.mark.parametrize("n", range(len(CASES)))
def test_random_shape(pgk, oracle, n):
    dtype, M, N, K, batch = CASES[n]
    rng = np.random.default_rng(1000 + n)
    call = CALLS[(n // 6) % 4]      # every size class meets every call twice
    splits = int(rng.choice([0, 1, 2, 3, 5]))
    if splits > K:
        splits = 0
    what = f"case {n}: dtype {dtype} {M}x{N}x{K} batch {batch} {call} splits {splits}"
    # integer-valued, identity: exact
    A, B = gen.make_int_inputs(dtype, M, N, K, batch, seed=n)
    ref_c, ref_rs = oracle.gemm_fused(A, B, None, gen.ACT_NONE)
    if dtype == BF16:
        ref_c = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref_c.astype(np.float32))).astype(np.float64)
    got_c, got_rs = run(pgk, call, A, B, None, gen.ACT_NONE, dtype, True, splits)
    assert np.array_equal(got_c, ref_c), what + " (integers): C"
    assert np.array_equal(got_rs, ref_rs), what + " (integers): rowsum"
    # random values, a random epilogue
    act = ACTS[int(rng.integers(4))]
    with_bias, with_rowsum = bool(rng.integers(2)), bool(rng.integers(2))
    A = gen.uniform(gen.tensor_seed(95, 1, n), batch * M * K, -1.0, 1.0).reshape(batch, M, K)
    B = gen.uniform(gen.tensor_seed(95, 2, n), batch * K * N, -1.0, 1.0).reshape(batch, K, N)
    bias = gen.normal(gen.tensor_seed(95, 3, n), N, 0.5) if with_bias else None
    if dtype == BF16:
        A, B = gen.f32_to_bf16_bits(A), gen.f32_to_bf16_bits(B)
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, act, want_rowsum=with_rowsum)
    got_c, got_rs = run(pgk, call, A, B, bias, act, dtype, with_rowsum, splits)
    e = rel_err(got_c, ref_c)
    assert e <= TOL[dtype], f"{what} act {act} bias {with_bias}: C error {e:.3e}"
    if with_rowsum:
        e = rel_err(got_rs, ref_rs)
        assert e <= TOL[dtype], f"{what} act {act} bias {with_bias}: rowsum error {e:.3e}"
    else:
        assert got_rs is None


def test_cases_reach_every_path(pgk):
    """The drawn shapes do cover what they are meant to: every tile shape of both types, the
    bounds-checked kernel and the automatic split (asked of the library's own plan query)."""
    seen = set()
    for n, (dtype, M, N, K, batch) in enumerate(CASES):
        p = pgk.gemm_plan(M, N, K, batch, dtype)
        seen.add((dtype, p["matrix_core"], p["tile"][:2], p["slices"] > 1))
        if p["tile"][:2] in ((256, 128), (128, 256)):     # which layout of B the half-tile cases run with
            call = CALLS[(n // 6) % 4]
            seen.add(("half tile, transposed B" if call.endswith("_bt") else "half tile, plain B", p["tile"][:2]))
    assert {("half tile, transposed B", (256, 128)), ("half tile, transposed B", (128, 256)),
            ("half tile, plain B", (256, 128)), ("half tile, plain B", (128, 256))} <= seen
    seen = {s for s in seen if len(s) == 4}
    tiles = {(d, t) for d, mc, t, s in seen if mc}
    assert {(F32, (128, 128)), (F32, (64, 64)), (BF16, (256, 256)), (BF16, (128, 128)), (BF16, (256, 128)), (BF16, (128, 256))} <= tiles
    assert any(not mc for d, mc, t, s in seen) and any(s for d, mc, t, s in seen)
