"""HIP graph capture of the library's calls (through torch's graph API, which only supplies
the capture stream): a call records kernel launches only -- the library allocates nothing, keeps
no state and records no memset node -- so the very first call of a shape on a stream can be
captured, with the workspace handed in by the caller, and each replay gives the bits of the
eager call on the inputs then in place."""
import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen
from util import to_device

pytestmark = pytest.mark.gpu

F32, BF16 = gen.F32, gen.BF16


@pytest.fixture(scope="module")
def pgk():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2511_06345_amd import binding
    binding.load_library()
    return binding


def _case(dtype, M, N, K, batch, seed):
    A = gen.uniform(gen.tensor_seed(93, 1, seed), batch * M * K, -1.0, 1.0).reshape(batch, M, K)
    B = gen.uniform(gen.tensor_seed(93, 2, seed), batch * K * N, -1.0, 1.0).reshape(batch, K, N)
    if dtype == BF16:
        A, B = gen.f32_to_bf16_bits(A), gen.f32_to_bf16_bits(B)
    return to_device(A, dtype), to_device(B, dtype)


# (dtype, M, N, K, batch, call): row sums over several tile columns (small grid, large grid), the
# automatic split of the fused call, the explicit split call, the bounds-checked kernel, and
# operands with rows off the 4-byte grid (copied into the workspace first)
CASES = [(F32, 256, 256, 256, 1, "fused"), (BF16, 1024, 1024, 512, 2, "fused"), (BF16, 64, 2048, 4096, 1, "fused"),
         (F32, 128, 128, 4096, 4, "splitk"), (F32, 13, 11, 100, 2, "fused"), (BF16, 130, 251, 515, 1, "fused")]


@pytest.mark.parametrize("case", CASES)
def test_first_call_is_capturable_and_replays_match_eager(pgk, case):
    import torch
    dtype, M, N, K, batch, call = case
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32
    bias = torch.from_numpy(gen.normal(gen.tensor_seed(93, 3, 0), N, 0.5)).cuda()
    inputs = [_case(dtype, M, N, K, batch, seed) for seed in range(3)]
    sA, sB = torch.empty_like(inputs[0][0]), torch.empty_like(inputs[0][1])
    C = torch.empty((batch, M, N), dtype=tdt, device="cuda")
    rs = torch.empty((batch, M), dtype=torch.float32, device="cuda")
    need = (pgk.gemm_splitk_workspace_bytes(M, N, K, batch, dtype, 0, pgk.WS_ROWSUM) if call == "splitk"
            else pgk.gemm_fused_workspace_bytes(M, N, K, batch, dtype, pgk.WS_ROWSUM))
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")     # the caller's, allocated before capture

    def launch(a, b, c, r, stream=None):
        if call == "splitk":
            pgk.gemm_splitk(a, b, bias, gen.ACT_GELU_TANH, splits=0, out=c, rowsum_out=r, workspace=ws, stream=stream)
        else:
            pgk.gemm_fused(a, b, bias, gen.ACT_GELU_TANH, out=c, rowsum_out=r, workspace=ws if need else None,
                           stream=stream)

    # capture first: nothing of this shape has run on this (new) stream, or anywhere, before
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        launch(sA, sB, C, rs, stream=side)
    # eager results on the default stream, own outputs, same workspace (the calls are ordered by
    # the synchronisations)
    eager = []
    for a, b in inputs:
        c, r = torch.empty_like(C), torch.empty_like(rs)
        launch(a, b, c, r)
        torch.cuda.synchronize()
        eager.append((c, r))
    view = torch.int16 if dtype == BF16 else torch.int32
    for rep in range(2):
        for i, (a, b) in enumerate(inputs):
            sA.copy_(a); sB.copy_(b)
            C.zero_(); rs.zero_()
            ws.fill_(0xFF)                  # whatever the workspace holds must not matter
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(C.view(view), eager[i][0].view(view)), f"replay {rep}/{i}: C differs from the eager call"
            assert torch.equal(rs, eager[i][1]), f"replay {rep}/{i}: row sums differ"
