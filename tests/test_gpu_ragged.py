"""GPU parity for GEMM shapes off the 16-byte grid and for very few rows: K or N not a multiple
of 4 (fp32) / 8 (bf16) elements -- the library copies the operands whose rows are not whole
16-byte chunks into zero-padded buffers and runs the matrix-core kernels on those, which store
output rows of any length -- and M below 16.  Every call (fused, split, either layout of B),
integer-valued inputs exactly, random ones within 1e-4 (fp32) / 2e-2 (bf16), what lies around the
output untouched.
"""
import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen
from util import TOL, c_to_numpy, rel_err, to_device

pytestmark = pytest.mark.gpu

F32, BF16 = gen.F32, gen.BF16
CALLS = ["fused", "fused_bt", "splitk", "splitk_bt"]

# (M, N, K, batch): ragged K, ragged even N, odd N, both, few rows, a partial last K tile on top,
# several tiles each way, a long K that the fused call splits by itself, outputs below 16 x 16
# with a long K, outputs of at most 32 columns or rows (the skinny tiles; a plain B of few columns
# is transposed first)
SHAPES = [(128, 128, 68, 1), (128, 132, 64, 1), (200, 301, 64, 2), (130, 250, 77, 3), (1, 512, 515, 1),
          (8, 1024, 1024, 1), (15, 260, 130, 2), (300, 1030, 129, 1), (640, 515, 70, 1), (64, 101, 4099, 1),
          (3, 17, 8200, 2), (513, 258, 1026, 1), (12, 12, 20000, 1), (8, 8, 1024, 3), (5, 3, 40002, 2),
          (300, 16, 1000, 2), (1000, 1, 515, 1), (257, 32, 4100, 1), (4096, 8, 64, 1), (100, 31, 333, 3), (32, 300, 520, 2),
          (2000, 24, 8192, 1), (20, 2000, 8192, 1),
          # one tile column or row, whole K tiles: K loops that start at a tile of their own (per tile, per batch entry)
          (512, 64, 1024, 3), (700, 128, 2048, 2), (40, 900, 1024, 3), (1100, 100, 512, 1), (2000, 32, 4096, 2)]


@pytest.fixture(scope="module")
def pgk():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2511_06345_amd import binding
    binding.load_library()
    return binding


def run(pgk, call, A, B, bias, act, dtype, rowsum, splits=0):
    """C and row sums, computed into the middle of larger buffers filled with a marker; also
    checks that the marker around them is untouched."""
    import torch
    bt = call.endswith("_bt")
    batch, M, K = A.shape
    N = B.shape[2]
    if bt:
        B = np.ascontiguousarray(np.swapaxes(B, 1, 2))
    dA, dB = to_device(A, dtype), to_device(B, dtype)
    dbias = torch.from_numpy(bias).cuda() if bias is not None else None
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32
    guard = 64                                       # elements; keeps C on the 16-byte grid
    flat = torch.full((batch * M * N + 2 * guard,), 7.0, dtype=tdt, device="cuda")
    C = flat[guard:guard + batch * M * N].view(batch, M, N)
    if call.startswith("fused"):
        C, rs = pgk.gemm_fused(dA, dB, dbias, act, rowsum=rowsum, b_transposed=bt, out=C)
    else:
        C, rs = pgk.gemm_splitk(dA, dB, dbias, act, splits=splits, rowsum=rowsum, b_transposed=bt, out=C)
    torch.cuda.synchronize()
    assert bool((flat[:guard] == 7.0).all()) and bool((flat[guard + batch * M * N:] == 7.0).all()), "wrote outside C"
    return c_to_numpy(C, dtype), (rs.cpu().numpy().astype(np.float64) if rs is not None else None)


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("call", CALLS)
@pytest.mark.parametrize("shape", SHAPES)
def test_ragged_shapes(pgk, oracle, dtype, call, shape):
    M, N, K, batch = shape
    n = SHAPES.index(shape)
    what = f"dtype {dtype} {M}x{N}x{K} batch {batch} {call}"
    A, B = gen.make_int_inputs(dtype, M, N, K, batch, seed=300 + n)
    ref_c, ref_rs = oracle.gemm_fused(A, B, None, gen.ACT_NONE)
    if dtype == BF16:
        ref_c = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref_c.astype(np.float32))).astype(np.float64)
    got_c, got_rs = run(pgk, call, A, B, None, gen.ACT_NONE, dtype, True, splits=[0, 3][n % 2])
    assert np.array_equal(got_c, ref_c), what + " (integers): C"
    assert np.array_equal(got_rs, ref_rs), what + " (integers): rowsum"

    act = [gen.ACT_SILU, gen.ACT_GELU_TANH, gen.ACT_RELU, gen.ACT_NONE][n % 4]
    A = gen.uniform(gen.tensor_seed(96, 1, n), batch * M * K, -1.0, 1.0).reshape(batch, M, K)
    B = gen.uniform(gen.tensor_seed(96, 2, n), batch * K * N, -1.0, 1.0).reshape(batch, K, N)
    bias = gen.normal(gen.tensor_seed(96, 3, n), N, 0.5)
    if dtype == BF16:
        A, B = gen.f32_to_bf16_bits(A), gen.f32_to_bf16_bits(B)
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, act, want_rowsum=True)
    got_c, got_rs = run(pgk, call, A, B, bias, act, dtype, True, splits=[0, 2][n % 2])
    e = rel_err(got_c, ref_c)
    assert e <= TOL[dtype], f"{what} act {act}: C error {e:.3e}"
    e = rel_err(got_rs, ref_rs)
    assert e <= TOL[dtype], f"{what} act {act}: rowsum error {e:.3e}"


def test_ragged_shapes_run_on_the_matrix_cores(pgk):
    """The plan query reports the matrix-core kernels for these shapes and for the sizes of real
    layers with awkward extents."""
    for dtype in (F32, BF16):
        for M, N, K, batch in SHAPES:
            p = pgk.gemm_plan(M, N, K, batch, dtype)
            assert p["matrix_core"], (dtype, M, N, K, p)
        for M, N, K in [(4096, 4096, 4100), (4096, 4100, 4096), (4096, 50257, 1024), (512, 30522, 768), (1, 4096, 4096), (8, 4096, 4096)]:
            assert pgk.gemm_plan(M, N, K, 1, dtype)["matrix_core"], (dtype, M, N, K)
        # the skinny tiles: flat for few rows, narrow for few columns (either layout of B)
        bk = 64 if dtype == BF16 else 32
        for bt in (False, True):
            assert pgk.gemm_plan(20, 2000, 8192, 1, dtype, b_transposed=bt)["tile"] == (32, 128, bk)
            assert pgk.gemm_plan(2000, 24, 8192, 1, dtype, b_transposed=bt)["tile"] == (128, 32, bk)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_vocabulary_sized_output_sampled_rows(pgk, oracle, dtype):
    """A projection onto an odd vocabulary size at full size: 512 x 30522 x 768 is fine for the
    oracle; 2048 x 50257 x 1024 is checked on sampled rows."""
    import torch
    for (M, N, K), rows in (((512, 30522, 768), None), ((2048, 50257, 1024), [0, 1, 255, 256, 1023, 2047])):
        A = gen.uniform(gen.tensor_seed(97, 1, N), M * K, -1.0, 1.0).reshape(1, M, K)
        B = gen.uniform(gen.tensor_seed(97, 2, N), K * N, -1.0, 1.0).reshape(1, K, N)
        bias = gen.normal(gen.tensor_seed(97, 3, N), N, 0.5)
        if dtype == BF16:
            A, B = gen.f32_to_bf16_bits(A), gen.f32_to_bf16_bits(B)
        dA, dB = to_device(A, dtype), to_device(B, dtype)
        C, rs = pgk.gemm_fused(dA, dB, torch.from_numpy(bias).cuda(), gen.ACT_SILU, rowsum=True)
        torch.cuda.synchronize()
        got_c, got_rs = c_to_numpy(C, dtype), rs.cpu().numpy().astype(np.float64)
        sel = np.arange(M) if rows is None else np.array(rows)
        ref_c, ref_rs = oracle.gemm_fused(A[:, sel], B, bias, gen.ACT_SILU, want_rowsum=True)
        e = rel_err(got_c[:, sel], ref_c)
        assert e <= TOL[dtype], f"dtype {dtype} {M}x{N}x{K}: C error {e:.3e}"
        e = rel_err(got_rs[:, sel], ref_rs)
        assert e <= TOL[dtype], f"dtype {dtype} {M}x{N}x{K}: rowsum error {e:.3e}"


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("call", CALLS)
@pytest.mark.parametrize("shape", [(130, 250, 78, 2), (64, 130, 4100, 1), (257, 66, 322, 3), (300, 258, 64, 1)])
def test_rows_read_in_place_ignore_their_surroundings(pgk, oracle, dtype, call, shape):
    """Rows that start on 4-byte boundaries but are not whole 16-byte chunks are read where they
    are: the last chunk of a row runs into the next row and, at the end of an operand, into
    whatever follows it in memory.  With NaNs right before and after A and B the result must
    still be exact (integer-valued inputs), down to the last row and column."""
    import torch
    M, N, K, batch = shape
    A, B = gen.make_int_inputs(dtype, M, N, K, batch, seed=500 + M)
    ref_c, ref_rs = oracle.gemm_fused(A, B, None, gen.ACT_NONE)
    if dtype == BF16:
        ref_c = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref_c.astype(np.float32))).astype(np.float64)
    bt = call.endswith("_bt")
    if bt:
        B = np.ascontiguousarray(np.swapaxes(B, 1, 2))
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32

    def inside_nans(arr):
        t = to_device(arr, dtype)
        flat = torch.full((t.numel() + 128,), float("nan"), dtype=tdt, device="cuda")
        flat[64:64 + t.numel()] = t.reshape(-1)
        return flat[64:64 + t.numel()].view(t.shape)

    dA, dB = inside_nans(A), inside_nans(B)
    if call.startswith("fused"):
        C, rs = pgk.gemm_fused(dA, dB, None, gen.ACT_NONE, rowsum=True, b_transposed=bt)
    else:
        C, rs = pgk.gemm_splitk(dA, dB, None, gen.ACT_NONE, splits=2, rowsum=True, b_transposed=bt)
    torch.cuda.synchronize()
    got_c, got_rs = c_to_numpy(C, dtype), rs.cpu().numpy().astype(np.float64)
    assert np.array_equal(got_c, ref_c), f"dtype {dtype} {shape} {call}: C"
    assert np.array_equal(got_rs, ref_rs), f"dtype {dtype} {shape} {call}: rowsum"
