"""HIP graph capture of the library's calls (through torch's graph API, which only supplies
the capture stream): every launch of a warmed-up call is capturable -- no allocation, no
memset node -- and each replay gives the bits of the eager call on the inputs then in place."""
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


# (dtype, M, N, K, batch, call): row sums combined inside the kernel (small grid), by the
# second kernel (large grid), the automatic split of the fused call, the explicit split call,
# the bounds-checked kernel
CASES = [(F32, 256, 256, 256, 1, "fused"), (BF16, 1024, 1024, 512, 2, "fused"), (BF16, 64, 2048, 4096, 1, "fused"),
         (F32, 128, 128, 4096, 4, "splitk"), (F32, 13, 11, 100, 2, "fused")]


@pytest.mark.parametrize("case", CASES)
def test_replays_match_eager(pgk, case):
    import torch
    dtype, M, N, K, batch, call = case
    tdt = torch.bfloat16 if dtype == BF16 else torch.float32
    bias = torch.from_numpy(gen.normal(gen.tensor_seed(93, 3, 0), N, 0.5)).cuda()
    inputs = [_case(dtype, M, N, K, batch, seed) for seed in range(3)]
    sA, sB = torch.empty_like(inputs[0][0]), torch.empty_like(inputs[0][1])
    C = torch.empty((batch, M, N), dtype=tdt, device="cuda")
    rs = torch.empty((batch, M), dtype=torch.float32, device="cuda")
    ws = None
    if call == "splitk":
        ws = torch.empty(pgk.splitk_workspace_bytes(M, N, K, batch, dtype, 0), dtype=torch.uint8, device="cuda")

    def launch(a, b, c, r, stream=None):
        if call == "splitk":
            pgk.gemm_splitk(a, b, bias, gen.ACT_GELU_TANH, splits=0, out=c, rowsum_out=r, workspace=ws, stream=stream)
        else:
            pgk.gemm_fused(a, b, bias, gen.ACT_GELU_TANH, out=c, rowsum_out=r, stream=stream)

    # eager results (also warms the library's scratch buffers up on both streams in use)
    eager = []
    for a, b in inputs:
        c, r = torch.empty_like(C), torch.empty_like(rs)
        launch(a, b, c, r)
        torch.cuda.synchronize()
        eager.append((c, r))
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        sA.copy_(inputs[0][0]); sB.copy_(inputs[0][1])
        launch(sA, sB, C, rs, stream=side)       # scratch for this stream exists before capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        launch(sA, sB, C, rs, stream=side)
    view = torch.int16 if dtype == BF16 else torch.int32
    for rep in range(2):
        for i, (a, b) in enumerate(inputs):
            sA.copy_(a); sB.copy_(b)
            C.zero_(); rs.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(C.view(view), eager[i][0].view(view)), f"replay {rep}/{i}: C differs from the eager call"
            assert torch.equal(rs, eager[i][1]), f"replay {rep}/{i}: row sums differ"
