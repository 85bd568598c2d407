"""GPU parity on seeded random skinny and ragged shapes: outputs with a few rows or columns (the
flat and narrow tiles, K in slices, a narrow B transposed first), outputs below 40 x 40 with a
long K, mid-size outputs with K and N off the 16-byte grid (rows read in place or copied), and K a
whole number of K tiles (rotated K loops) -- every call, either layout of B, random slice counts.
Integer-valued inputs (entries in {-2..2}), so C and the row sums must match the oracle exactly.
"""
import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen
from util import c_to_numpy, to_device

pytestmark = pytest.mark.gpu

CALLS = ["fused", "fused_bt", "splitk", "splitk_bt"]


@pytest.fixture(scope="module")
def pgk():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2511_06345_amd import binding
    binding.load_library()
    return binding


def draw_cases(seed, count):
    rng = np.random.default_rng(seed)
    cases = []
    for n in range(count):
        dtype = gen.BF16 if rng.integers(2) else gen.F32
        cls = n % 5
        if cls == 0:
            M, N, K = int(rng.integers(1, 40)), int(rng.integers(1, 3000)), int(rng.integers(1, 9000))
        elif cls == 1:
            M, N, K = int(rng.integers(1, 3000)), int(rng.integers(1, 40)), int(rng.integers(1, 9000))
        elif cls == 2:
            M, N, K = int(rng.integers(1, 40)), int(rng.integers(1, 40)), int(rng.integers(1, 60000))
        elif cls == 3:
            M, N, K = int(rng.integers(100, 1500)), int(rng.integers(100, 1500)), int(rng.integers(1, 1500))
        else:
            M, N, K = int(rng.integers(1, 600)), int(rng.integers(1, 600)), 64 * int(rng.integers(1, 64))
        batch = int(rng.integers(1, 4))
        if M * N * K * batch > 2e9:                     # keeps the oracle at a second or so per case
            K = max(1, int(2e9 / (M * N * batch)))
        call = CALLS[int(rng.integers(4))]
        splits = int(rng.choice([0, 0, 2, 3, 7]))
        cases.append((dtype, M, N, K, batch, call, 0 if splits > K else splits))
    return cases


CASES = draw_cases(20251128, 70)


@pytest.mark.parametrize("n", range(len(CASES)))
def test_random_skinny_shape(pgk, oracle, n):
    import torch
    dtype, M, N, K, batch, call, splits = CASES[n]
    what = f"case {n}: dtype {dtype} {M}x{N}x{K} batch {batch} {call} splits {splits}"
    A, B = gen.make_int_inputs(dtype, M, N, K, batch, seed=n)
    ref_c, ref_rs = oracle.gemm_fused(A, B, None, gen.ACT_NONE)
    if dtype == gen.BF16:
        ref_c = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref_c.astype(np.float32))).astype(np.float64)
    bt = call.endswith("_bt")
    dA = to_device(A, dtype)
    dB = to_device(np.ascontiguousarray(np.swapaxes(B, 1, 2)) if bt else B, dtype)
    if call.startswith("fused"):
        C, rs = pgk.gemm_fused(dA, dB, None, gen.ACT_NONE, rowsum=True, b_transposed=bt)
    else:
        C, rs = pgk.gemm_splitk(dA, dB, None, gen.ACT_NONE, splits=splits, rowsum=True, b_transposed=bt)
    torch.cuda.synchronize()
    assert np.array_equal(c_to_numpy(C, dtype), ref_c), what + ": C"
    assert np.array_equal(rs.cpu().numpy().astype(np.float64), ref_rs), what + ": rowsum"


def test_cases_reach_the_skinny_tiles(pgk):
    seen = set()
    for dtype, M, N, K, batch, call, splits in CASES:
        p = pgk.gemm_plan(M, N, K, batch, dtype, b_transposed=call.endswith("_bt"))
        seen.add((dtype, p["matrix_core"], p["tile"][:2], p["slices"] > 1))
    for dtype in (gen.F32, gen.BF16):
        for tile in ((32, 128), (128, 32)):
            assert any(s[0] == dtype and s[2] == tile and s[3] for s in seen), (dtype, tile, "split")
