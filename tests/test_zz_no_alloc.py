"""pgk_gemm_fused_static -- the fused call for callers that cannot allocate -- against
pgk_gemm_fused with a caller workspace: same kernels, so the outputs must agree bit for bit,
on two calls in a row, the second on a smaller problem (the fixed array then still holds the
first call's partial row sums), and both must match the CPU oracle within the library's bar.
Runs last: it is the one test that touches the library's fixed device array."""
import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen
from util import TOL, c_to_numpy, rel_err, to_device

pytestmark = pytest.mark.gpu

F32, BF16 = gen.F32, gen.BF16


@pytest.fixture(scope="module")
def pgk():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2511_06345_amd import binding
    binding.load_library()
    return binding


def _inputs(dtype, M, N, K, batch, seed):
    A = gen.uniform(gen.tensor_seed(96, 1, seed), batch * M * K, -1.0, 1.0).reshape(batch, M, K)
    B = gen.uniform(gen.tensor_seed(96, 2, seed), batch * K * N, -1.0, 1.0).reshape(batch, K, N)
    bias = gen.normal(gen.tensor_seed(96, 3, seed), N, 0.5)
    if dtype == BF16:
        A, B = gen.f32_to_bf16_bits(A), gen.f32_to_bf16_bits(B)
    return A, B, bias


# (dtype, first problem, second and smaller problem): each needs the workspace -- row sums over
# several tile columns -- and the third pair also an automatic K split and operand copies
PAIRS = [(BF16, (2048, 1024, 512, 1), (300, 520, 200, 2)),
         (F32, (256, 256, 256, 1), (70, 130, 36, 3)),
         (BF16, (64, 512, 4096, 1), (130, 251, 515, 1))]


@pytest.mark.parametrize("pair", PAIRS)
def test_static_entry_matches_the_workspace_call(pgk, oracle, pair):
    import torch
    dtype, first, second = pair
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32
    view = torch.int16 if dtype == BF16 else torch.int32
    limit = pgk.gemm_fused_static_max_bytes()
    assert limit == 4 << 20
    for n, (M, N, K, batch) in enumerate((first, second)):
        need = pgk.gemm_fused_workspace_bytes(M, N, K, batch, dtype, pgk.WS_ROWSUM)
        assert 0 < need <= limit, (M, N, K, batch, need)
        A, B, bias = _inputs(dtype, M, N, K, batch, seed=17 * n + M)
        dA, dB, dbias = to_device(A, dtype), to_device(B, dtype), torch.from_numpy(bias).cuda()
        act = gen.ACT_SILU if n == 0 else gen.ACT_GELU_TANH
        # the existing entry point, workspace from the caller
        C_ref, rs_ref = pgk.gemm_fused(dA, dB, dbias, act, rowsum=True)
        # the new one: outputs only
        C = torch.full((batch, M, N), -3.0, dtype=tdt, device="cuda")
        rs = torch.full((batch, M), -3.0, dtype=torch.float32, device="cuda")
        pgk.gemm_fused_static(dA, dB, dbias, act, out=C, rowsum_out=rs)
        torch.cuda.synchronize()
        assert torch.equal(C.view(view), C_ref.view(view)), f"call {n}: C differs from pgk_gemm_fused"
        assert torch.equal(rs.view(torch.int32), rs_ref.view(torch.int32)), f"call {n}: row sums differ"
        ref_c, ref_rs = oracle.gemm_fused(A, B, bias, act)
        assert rel_err(c_to_numpy(C, dtype), ref_c) <= TOL[dtype]
        assert rel_err(rs.cpu().numpy().astype(np.float64), ref_rs) <= TOL[dtype]


def test_static_entry_refuses_what_does_not_fit(pgk):
    import torch
    # an automatic K split whose partial products exceed the fixed array: refused on the host
    M, N, K = 1024, 1024, 8192
    assert pgk.gemm_fused_workspace_bytes(M, N, K, 1, BF16, 0) > pgk.gemm_fused_static_max_bytes()
    a = torch.zeros((1, M, K), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((1, K, N), dtype=torch.bfloat16, device="cuda")
    c = torch.full((1, M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(pgk.PgkError) as ei:
        pgk.gemm_fused_static(a, b, None, gen.ACT_NONE, out=c)
    assert ei.value.status == -3
    torch.cuda.synchronize()
    assert bool((c == 7.0).all()), "a refused call must not have launched anything"
    # a problem that needs no workspace at all runs without touching the array
    a = torch.ones((1, 256, 64), dtype=torch.bfloat16, device="cuda")
    b = torch.ones((1, 64, 256), dtype=torch.bfloat16, device="cuda")
    c = torch.empty((1, 256, 256), dtype=torch.bfloat16, device="cuda")
    assert pgk.gemm_fused_workspace_bytes(256, 256, 64, 1, BF16, 0) == 0
    pgk.gemm_fused_static(a, b, None, gen.ACT_NONE, out=c)
    torch.cuda.synchronize()
    assert bool((c == 64.0).all())
