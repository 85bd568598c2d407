"""GPU parity of the calls that take the second factor transposed (Bt [batch][N][K], read in
place): pgk_gemm_fused_bt / pgk_gemm_splitk_bt against the CPU oracle's C = act(A Bt^T + bias).

Same bars as for the plain calls: 1e-4 (fp32) / 2e-2 (bf16) on max |g - r| / max(|r|, RMS(r));
integer-valued inputs with the identity activation must match exactly.
"""
import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen
from util import TOL, c_to_numpy, rel_err, sample_rows, to_device

pytestmark = pytest.mark.gpu

NONE, RELU, GELU, SILU = gen.ACT_NONE, gen.ACT_RELU, gen.ACT_GELU_TANH, gen.ACT_SILU
F32, BF16 = gen.F32, gen.BF16


@pytest.fixture(scope="module")
def pgk():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2511_06345_amd import binding
    binding.load_library()
    return binding


def run_bt(pgk, A, Bt, bias, act, dtype, rowsum=True, splits=None):
    import torch
    dA, dB = to_device(A, dtype), to_device(Bt, dtype)
    dbias = torch.from_numpy(bias).cuda() if bias is not None else None
    if splits is None:
        C, rs = pgk.gemm_fused_bt(dA, dB, dbias, act, rowsum=rowsum)
    else:
        C, rs = pgk.gemm_splitk_bt(dA, dB, dbias, act, splits=splits, rowsum=rowsum)
    torch.cuda.synchronize()
    return c_to_numpy(C, dtype), (rs.cpu().numpy().astype(np.float64) if rs is not None else None)


def random_case(dtype, M, N, K, batch, seed, bias_std=0.5):
    A = gen.uniform(gen.tensor_seed(91, 1, seed), batch * M * K, -1.0, 1.0).reshape(batch, M, K)
    Bt = gen.uniform(gen.tensor_seed(91, 2, seed), batch * N * K, -1.0, 1.0).reshape(batch, N, K)
    bias = gen.normal(gen.tensor_seed(91, 3, seed), N, bias_std)
    if dtype == BF16:
        A, Bt = gen.f32_to_bf16_bits(A), gen.f32_to_bf16_bits(Bt)
    return A, Bt, bias


def int_case(dtype, M, N, K, batch, seed):
    A, B = gen.make_int_inputs(dtype, M, N, K, batch, seed=seed)
    return A, np.ascontiguousarray(np.swapaxes(B, 1, 2))


def check(got_c, got_rs, ref_c, ref_rs, dtype, what):
    e = rel_err(got_c, ref_c)
    assert e <= TOL[dtype], f"{what}: C error {e:.3e}"
    if ref_rs is not None and got_rs is not None:
        e = rel_err(got_rs, ref_rs)
        assert e <= TOL[dtype], f"{what}: rowsum error {e:.3e}"


def bf16_round(ref):
    return gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref.astype(np.float32))).astype(np.float64)


# bounds-checked kernel (tiny / odd sizes); matrix-core kernels on the small tiles (exact
# multiples, ragged M and N, partial last K tile) and, with many batch entries, on the large ones
GUARDED = [(1, 1, 1, 1), (5, 7, 33, 2), (65, 63, 17, 1), (130, 70, 100, 3), (2, 300, 5, 1), (15, 15, 1000, 2), (9, 14, 513, 3), (33, 31, 255, 1)]
SMALL_TILE = {F32: [(128, 128, 32, 1), (128, 384, 160, 2), (100, 36, 64, 2), (129, 132, 96, 1), (17, 500, 128, 1),
                    (250, 16, 64, 3), (128, 128, 36, 1), (100, 36, 4, 2), (70, 200, 524, 1)],
              BF16: [(256, 256, 64, 1), (512, 256, 320, 2), (100, 40, 64, 2), (257, 264, 128, 1), (17, 1000, 192, 1),
                     (700, 16, 64, 2), (256, 256, 72, 1), (100, 40, 8, 2), (130, 72, 1032, 1)]}
LARGE_TILE = {F32: [(128, 128, 32, 192), (300, 260, 64, 40), (129, 140, 300, 70)],
              BF16: [(256, 256, 64, 192), (300, 520, 128, 40), (257, 264, 520, 50), (256, 256, 1032, 48)]}


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("act", [NONE, RELU, GELU, SILU])
def test_random_inputs(pgk, oracle, dtype, act):
    for shape in GUARDED + SMALL_TILE[dtype] + LARGE_TILE[dtype][:2]:
        M, N, K, batch = shape
        A, Bt, bias = random_case(dtype, M, N, K, batch, seed=M + 3 * N + 7 * K)
        ref_c, ref_rs = oracle.gemm_fused_bt(A, Bt, bias, act)
        got_c, got_rs = run_bt(pgk, A, Bt, bias, act, dtype)
        check(got_c, got_rs, ref_c, ref_rs, dtype, f"{shape} act {act}")
        ref_c, _ = oracle.gemm_fused_bt(A, Bt, None, act, want_rowsum=False)
        got_c, got_rs = run_bt(pgk, A, Bt, None, act, dtype, rowsum=False)
        assert got_rs is None
        check(got_c, None, ref_c, None, dtype, f"{shape} act {act} no bias")


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_integer_inputs_are_exact(pgk, oracle, dtype):
    """Entries in {-2..2}, identity: exact for every tile path and K-tile count, fused and split."""
    for shape in GUARDED + SMALL_TILE[dtype] + LARGE_TILE[dtype]:
        M, N, K, batch = shape
        A, Bt = int_case(dtype, M, N, K, batch, seed=11 * M + K)
        ref_c, ref_rs = oracle.gemm_fused_bt(A, Bt, None, NONE)
        if dtype == BF16:
            ref_c = bf16_round(ref_c)
        got_c, got_rs = run_bt(pgk, A, Bt, None, NONE, dtype)
        assert np.array_equal(got_c, ref_c), f"fused {shape}"
        assert np.array_equal(got_rs, ref_rs), f"fused rowsum {shape}"
        for splits in (0, 1, 3):
            if splits > K:
                continue
            got_c, got_rs = run_bt(pgk, A, Bt, None, NONE, dtype, splits=splits)
            assert np.array_equal(got_c, ref_c), f"split {shape} splits {splits}"
            assert np.array_equal(got_rs, ref_rs), f"split rowsum {shape} splits {splits}"


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_skinny_and_long_k(pgk, oracle, dtype):
    """Shapes the fused call splits by itself (few tiles, long K), and the split call with
    explicit counts; deterministic from run to run."""
    for shape in [(16, 4096, 512, 1), (40, 1288, 2048, 2), (256, 256, 4096, 1), (100, 36, 1000, 2)]:
        M, N, K, batch = shape
        A, Bt, bias = random_case(dtype, M, N, K, batch, seed=5 * M + K)
        ref_c, ref_rs = oracle.gemm_fused_bt(A, Bt, bias, SILU)
        got_c, got_rs = run_bt(pgk, A, Bt, bias, SILU, dtype)
        check(got_c, got_rs, ref_c, ref_rs, dtype, f"fused {shape}")
        for splits in (0, 4, 7):
            c1, r1 = run_bt(pgk, A, Bt, bias, SILU, dtype, splits=splits)
            check(c1, r1, ref_c, ref_rs, dtype, f"split {shape} splits {splits}")
            c2, r2 = run_bt(pgk, A, Bt, bias, SILU, dtype, splits=splits)
            assert np.array_equal(c1, c2) and np.array_equal(r1, r2)


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("batch", [2, 48])
def test_k_tail_ignores_what_follows_a_row(pgk, oracle, dtype, batch):
    """K not a multiple of the K tile: the missing columns of the last K tile lie, in memory,
    over the start of the next row of A and of Bt, and after the last row over whatever follows
    the array.  NaNs planted there must not reach the rows / columns before them."""
    import torch
    M, N, K = 260, 264, 200 if dtype == BF16 else 100
    A, Bt, bias = random_case(dtype, M, N, K, batch, seed=78)
    ref_c, _ = oracle.gemm_fused_bt(A, Bt, bias, NONE, want_rowsum=False)
    nan = np.uint16(0x7FC0) if dtype == BF16 else np.float32(np.nan)
    bad_row, bad_col = 131, 77
    A2, B2 = A.copy(), Bt.copy()
    A2[:, bad_row, :16] = nan
    B2[:, bad_col, :16] = nan
    # the arrays handed to the library are the first `batch` entries of larger ones whose
    # last entry is all NaN: that is what lies behind the last row
    A3 = np.concatenate([A2, np.full((1, M, K), nan, dtype=A2.dtype)])
    B3 = np.concatenate([B2, np.full((1, N, K), nan, dtype=B2.dtype)])
    dA, dB = to_device(A3, dtype)[:batch], to_device(B3, dtype)[:batch]
    C, _ = pgk.gemm_fused_bt(dA, dB, torch.from_numpy(bias).cuda(), NONE, rowsum=False)
    torch.cuda.synchronize()
    got_c = c_to_numpy(C, dtype)
    keep = np.ones((batch, M, N), dtype=bool)
    keep[:, bad_row, :] = False
    keep[:, :, bad_col] = False
    assert np.all(np.isfinite(got_c[keep])), "a NaN leaked out of its row / column"
    assert np.all(np.isnan(got_c[~keep]))
    e = rel_err(got_c[keep], ref_c[keep])
    assert e <= TOL[dtype], f"C error {e:.3e}"


def test_linear_layer_shape_sampled_rows(pgk, oracle):
    """A large bf16 problem on the 256x256 tiles (tokens x features, weight [out][in]), bare
    product and with bias + SiLU, on sampled rows; bit-equal from run to run."""
    import torch
    M, N, K = 4096, 4096, 4096
    A = gen.f32_to_bf16_bits(gen.normal(gen.tensor_seed(92, 1, 0), M * K, 1.0).reshape(1, M, K))
    W = gen.f32_to_bf16_bits(gen.normal(gen.tensor_seed(92, 2, 0), N * K, 1.0 / 64).reshape(1, N, K))
    bias = gen.normal(gen.tensor_seed(92, 3, 0), N, 0.1)
    rows = sample_rows(M, 256, 32, seed=5)
    dA, dW, dbias = to_device(A, BF16), to_device(W, BF16), torch.from_numpy(bias).cuda()
    drows = torch.from_numpy(rows).cuda()
    for b, act in ((None, NONE), (bias, SILU)):
        ref_c, ref_rs = oracle.gemm_fused_bt(A, W, b, act, rows=rows)
        C, rs = pgk.gemm_fused_bt(dA, dW, dbias if b is not None else None, act)
        C2, rs2 = pgk.gemm_fused_bt(dA, dW, dbias if b is not None else None, act)
        torch.cuda.synchronize()
        assert torch.equal(C.view(torch.int16), C2.view(torch.int16)) and torch.equal(rs, rs2)
        check(c_to_numpy(C[:, drows], BF16), rs[:, drows].cpu().numpy().astype(np.float64), ref_c, ref_rs, BF16,
              f"linear layer act {act}")


def test_transposed_and_plain_calls_agree_exactly(pgk):
    """Same factors, two storage orders: both calls add the same products in the same order
    on the matrix-core path, so the results are bit-equal."""
    import torch
    for dtype, shape in ((F32, (300, 260, 100, 3)), (BF16, (300, 520, 200, 2))):
        M, N, K, batch = shape
        A, Bt, bias = random_case(dtype, M, N, K, batch, seed=3)
        B = np.ascontiguousarray(np.swapaxes(Bt, 1, 2))
        dbias = torch.from_numpy(bias).cuda()
        C1, r1 = pgk.gemm_fused_bt(to_device(A, dtype), to_device(Bt, dtype), dbias, GELU)
        C2, r2 = pgk.gemm_fused(to_device(A, dtype), to_device(B, dtype), dbias, GELU)
        torch.cuda.synchronize()
        assert np.array_equal(c_to_numpy(C1, dtype), c_to_numpy(C2, dtype)) and torch.equal(r1, r2)


def test_error_codes(pgk):
    import torch
    a = torch.zeros(1, 8, 8, device="cuda")
    with pytest.raises(pgk.PgkError) as ei:
        pgk.gemm_splitk_bt(a, a, None, NONE, splits=9)
    assert ei.value.status == -1
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(pgk.PgkError) as ei:
        pgk.gemm_splitk_bt(a, a, None, NONE, splits=1, workspace=small)
    assert ei.value.status == -3
    with pytest.raises(ValueError):
        pgk.gemm_fused_bt(torch.zeros(1, 8, 16, device="cuda"), torch.zeros(1, 8, 8, device="cuda"), None, NONE)
