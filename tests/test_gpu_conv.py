"""GPU parity of conv1d: the HIP path (through the C ABI) against the CPU oracle on the same
seeded inputs.  Error bar as for the GEMM it is computed by: max |g - r| / max(|r|, RMS(r))
<= 1e-4 for fp32 and <= 2e-2 for bf16 with fp32 accumulation; integer-valued inputs with the
identity activation must match exactly."""
import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen
from util import TOL, c_to_numpy, rel_err, to_device

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


def run(pgk, x, w, bias, act, dtype, stride, pad, dilation):
    import torch
    dx, dw = to_device(x, dtype), to_device(w, dtype)
    db = torch.from_numpy(bias).cuda() if bias is not None else None
    y = pgk.conv1d(dx, dw, db, act, stride, pad, dilation)
    torch.cuda.synchronize()
    return c_to_numpy(y, dtype)


def random_case(dtype, B, Cin, L, Cout, Kw, seed):
    x = gen.uniform(gen.tensor_seed(98, 1, seed), B * Cin * L, -1.0, 1.0).reshape(B, Cin, L)
    w = gen.uniform(gen.tensor_seed(98, 2, seed), Cout * Cin * Kw, -1.0, 1.0).reshape(Cout, Cin, Kw)
    bias = gen.normal(gen.tensor_seed(98, 3, seed), Cout, 0.5)
    if dtype == BF16:
        x, w = gen.f32_to_bf16_bits(x), gen.f32_to_bf16_bits(w)
    return x, w, bias


def int_case(dtype, B, Cin, L, Cout, Kw, seed):
    x = gen.small_ints(gen.tensor_seed(98, 4, seed), B * Cin * L).reshape(B, Cin, L)
    w = gen.small_ints(gen.tensor_seed(98, 5, seed), Cout * Cin * Kw).reshape(Cout, Cin, Kw)
    if dtype == BF16:
        x, w = gen.f32_to_bf16_bits(x), gen.f32_to_bf16_bits(w)
    return x, w


# (B, Cin, L, Cout, Kw, stride, pad, dilation).  FAST: enough channels, at least 16 output
# channels and outputs -> matrix-core path (shifted views, several taps, padded copy or not,
# small and large tiles, ragged Cout and Lout tiles, any output length).
FAST = {
    F32: [(2, 32, 256, 32, 3, 1, 1, 1), (1, 64, 1024, 48, 5, 1, 2, 1), (3, 32, 520, 130, 3, 1, 1, 1),
          (2, 96, 300, 64, 1, 1, 0, 1), (2, 32, 1028, 20, 4, 1, 3, 2), (1, 32, 1024, 64, 7, 1, 9, 3),
          (40, 64, 2048, 128, 3, 1, 1, 1), (2, 64, 4096, 256, 3, 1, 0, 2),
          # one tile column that is first and last at once; right edge spread over two tile columns;
          # padding wider than a tile (padded copy of the whole input); halo wider than a tile
          (2, 32, 60, 32, 5, 1, 2, 1), (2, 32, 1024, 32, 9, 1, 6, 1), (2, 32, 500, 32, 3, 1, 101, 1), (1, 32, 2000, 32, 5, 1, 0, 40),
          # stride > 1 (one copy of the input per phase), channel counts that are not a multiple of the K tile
          # (copies and weights padded with zero channels), both, large tiles
          (2, 64, 1000, 32, 3, 2, 1, 1), (2, 32, 1024, 48, 5, 2, 2, 1), (2, 32, 1200, 32, 4, 3, 2, 2), (2, 48, 1000, 32, 3, 1, 1, 1),
          (3, 80, 520, 130, 5, 1, 2, 1), (40, 96, 2048, 256, 3, 2, 1, 1), (2, 20, 4096, 64, 7, 4, 3, 1),
          # output lengths that are not a multiple of the 16-byte chunk, on every route
          (2, 32, 1001, 32, 3, 1, 0, 1), (2, 32, 1001, 40, 3, 1, 1, 1), (2, 64, 1000, 32, 3, 2, 0, 1), (2, 48, 777, 32, 5, 1, 2, 1),
          (3, 32, 101, 33, 3, 1, 1, 1), (2, 64, 257, 16, 3, 2, 1, 1), (2, 32, 1024, 32, 3, 1, 0, 1),
          # few output channels: the flat tile, on every route
          (2, 64, 256, 8, 3, 1, 1, 1), (3, 64, 1000, 1, 3, 1, 1, 1), (2, 32, 1001, 5, 5, 2, 2, 1), (2, 64, 4096, 20, 3, 1, 0, 2), (2, 48, 600, 3, 3, 1, 50, 1)],
    BF16: [(2, 64, 256, 32, 3, 1, 2, 2), (1, 128, 1024, 48, 5, 1, 4, 2), (3, 64, 520, 130, 1, 1, 0, 1),
           (2, 64, 1032, 24, 3, 1, 4, 4), (40, 128, 2048, 256, 3, 1, 2, 2), (2, 64, 4104, 256, 2, 1, 0, 8),
           (2, 64, 120, 32, 5, 1, 4, 2), (2, 64, 1030, 32, 3, 1, 3, 2), (2, 64, 1036, 32, 9, 1, 6, 2),
           # odd dilation: taps at odd column offsets come from a second copy shifted by one element
           (2, 64, 256, 32, 3, 1, 1, 1), (1, 128, 1024, 48, 5, 1, 2, 1), (3, 64, 519, 130, 2, 1, 1, 1), (40, 128, 2048, 256, 3, 1, 1, 1),
           (2, 64, 1032, 32, 3, 1, 3, 3), (2, 64, 1024, 32, 9, 1, 4, 1), (2, 64, 2004, 32, 5, 1, 0, 5), (2, 64, 504, 32, 3, 1, 101, 1),
           (2, 64, 1025, 32, 4, 1, 1, 1), (1, 64, 64, 16, 7, 1, 3, 1),
           # stride > 1, ragged channel counts, both with odd and even tap offsets
           (2, 64, 1024, 32, 3, 2, 1, 1), (2, 96, 1024, 32, 3, 1, 1, 1), (2, 64, 1200, 32, 4, 3, 2, 2), (40, 160, 2048, 256, 3, 2, 1, 1),
           (2, 64, 1040, 32, 5, 2, 6, 3), (2, 40, 4096, 64, 7, 4, 3, 1),
           # output lengths that are odd, or even and not a multiple of the chunk, on every route
           (2, 64, 1001, 32, 3, 1, 0, 2), (2, 64, 1001, 32, 3, 1, 1, 1), (2, 64, 1000, 32, 3, 2, 0, 1), (2, 64, 1030, 32, 3, 1, 0, 2),
           (3, 32, 101, 33, 3, 1, 1, 1), (2, 64, 257, 16, 3, 2, 1, 1), (2, 64, 1024, 32, 3, 1, 0, 2),
           (2, 64, 256, 8, 3, 1, 2, 2), (3, 64, 1000, 1, 3, 1, 1, 1), (2, 64, 1001, 5, 5, 2, 2, 1), (2, 64, 4096, 20, 3, 1, 0, 2), (2, 96, 600, 3, 3, 1, 50, 1)],
}
# everything else: the bounds-checked kernel reading the input in place
GENERAL = [(1, 1, 9, 1, 3, 1, 0, 1), (2, 3, 17, 4, 3, 1, 1, 1), (2, 5, 50, 7, 5, 2, 2, 1), (1, 2, 130, 70, 4, 3, 5, 2),
           (1, 7, 300, 5, 9, 1, 0, 3), (2, 64, 15, 8, 3, 1, 1, 1), (2, 8, 101, 33, 3, 1, 1, 1)]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("act", [NONE, SILU])
def test_matrix_core_path(pgk, oracle, dtype, act):
    for cfg in FAST[dtype]:
        B, Cin, L, Cout, Kw, stride, pad, dilation = cfg
        assert pgk.conv1d_workspace_bytes(B, Cin, L, Cout, Kw, stride, pad, dilation, dtype) > 0, cfg
        x, w, bias = random_case(dtype, B, Cin, L, Cout, Kw, seed=L + Kw)
        ref = oracle.conv1d(x, w, bias, act, stride, pad, dilation)
        got = run(pgk, x, w, bias, act, dtype, stride, pad, dilation)
        assert got.shape == ref.shape
        e = rel_err(got, ref)
        assert e <= TOL[dtype], f"{cfg} act {act}: error {e:.3e}"
        xi, wi = int_case(dtype, B, Cin, L, Cout, Kw, seed=L)
        ref = oracle.conv1d(xi, wi, None, NONE, stride, pad, dilation)
        got = run(pgk, xi, wi, None, NONE, dtype, stride, pad, dilation)
        if dtype == BF16:
            ref = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref.astype(np.float32))).astype(np.float64)
        assert np.array_equal(got, ref), f"{cfg}: integer inputs"


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("act", [NONE, RELU, GELU])
def test_general_path(pgk, oracle, dtype, act):
    for cfg in GENERAL:
        B, Cin, L, Cout, Kw, stride, pad, dilation = cfg
        assert pgk.conv1d_workspace_bytes(B, Cin, L, Cout, Kw, stride, pad, dilation, dtype) == 0, cfg
        x, w, bias = random_case(dtype, B, Cin, L, Cout, Kw, seed=L + 3 * Kw)
        ref = oracle.conv1d(x, w, bias, act, stride, pad, dilation)
        got = run(pgk, x, w, bias, act, dtype, stride, pad, dilation)
        e = rel_err(got, ref)
        assert e <= TOL[dtype], f"{cfg} act {act}: error {e:.3e}"
        xi, wi = int_case(dtype, B, Cin, L, Cout, Kw, seed=L)
        ref = oracle.conv1d(xi, wi, None, NONE, stride, pad, dilation)
        got = run(pgk, xi, wi, None, NONE, dtype, stride, pad, dilation)
        if dtype == BF16:
            ref = gen.bf16_bits_to_f32(gen.f32_to_bf16_bits(ref.astype(np.float32))).astype(np.float64)
        assert np.array_equal(got, ref), f"{cfg}: integer inputs"


def test_both_paths_agree_and_are_deterministic(pgk):
    """The same problem through the matrix-core path and, made ineligible by a misaligned
    input pointer, through the bounds-checked kernel."""
    import torch
    B, Cin, L, Cout, Kw = 2, 32, 512, 40, 3
    x, w = int_case(F32, B, Cin, L, Cout, Kw, seed=3)
    dx, dw = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    a = pgk.conv1d(dx, dw, None, NONE, 1, 1, 1)
    a2 = pgk.conv1d(dx, dw, None, NONE, 1, 1, 1)
    flat = torch.cat([torch.zeros(1, device="cuda"), dx.reshape(-1)])
    off = flat[1:].view(B, Cin, L)
    b = pgk.conv1d(off, dw, None, NONE, 1, 1, 1)
    # weights and output one element past a 16-byte boundary: still the matrix-core path (the
    # weights are regrouped into the workspace, output rows may start on any element)
    woff = torch.cat([torch.zeros(1, device="cuda"), dw.reshape(-1)])[1:].view(Cout, Cin, Kw)
    yflat = torch.full((a.numel() + 2,), 7.0, device="cuda")
    c = pgk.conv1d(dx, woff, None, NONE, 1, 1, 1, out=yflat[1:-1].view(a.shape))
    torch.cuda.synchronize()
    assert torch.equal(a, a2) and torch.equal(a, b) and torch.equal(a, c)
    assert float(yflat[0]) == 7.0 and float(yflat[-1]) == 7.0


@pytest.mark.parametrize("name", sorted(gen.CONV_WORKLOADS))
def test_conv_workloads_sampled(pgk, oracle, name):
    """The benchmark's convolution workloads at full size; the oracle evaluates a seeded sample
    of batch entries and output channels in full."""
    import torch
    cw = gen.CONV_WORKLOADS[name]
    x, w, bias = gen.make_conv_inputs(cw)
    dx, dw = to_device(x, cw.dtype), to_device(w, cw.dtype)
    y = pgk.conv1d(dx, dw, torch.from_numpy(bias).cuda(), cw.act, cw.stride, cw.pad, cw.dilation)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    bs = sorted(set([0, cw.B - 1] + rng.integers(0, cw.B, 1).tolist()))
    cos = sorted(set([0, cw.Cout - 1] + rng.integers(0, cw.Cout, 6).tolist()))
    for b in bs:
        ref = oracle.conv1d(x[b:b + 1], w[cos], bias[cos], cw.act, cw.stride, cw.pad, cw.dilation)[0]
        got = c_to_numpy(y[b][cos], cw.dtype)
        e = rel_err(got, ref)
        assert e <= TOL[cw.dtype], f"{name} batch {b}: error {e:.3e}"


def test_input_larger_than_4_gib(pgk, oracle):
    """x [132, 256, 65536] bf16 = 4.4 GB, one seeded batch entry repeated: byte offsets of the
    later entries exceed 32 bits.  Matrix-core path (stride 1, padded, dilated); every entry
    must equal the oracle's result for the one entry, on sampled output channels."""
    import torch
    B, Cin, L, Cout, Kw, pad, dil = 132, 256, 65536, 64, 3, 2, 2
    x1, w, bias = random_case(BF16, 1, Cin, L, Cout, Kw, seed=77)
    dx = to_device(x1, BF16).expand(B, -1, -1).contiguous()
    assert dx.numel() * 2 > (1 << 32)
    y = pgk.conv1d(dx, to_device(w, BF16), torch.from_numpy(bias).cuda(), RELU, 1, pad, dil)
    torch.cuda.synchronize()
    assert pgk.conv1d_workspace_bytes(B, Cin, L, Cout, Kw, 1, pad, dil, BF16) > 0, "expected the matrix-core path"
    ref = oracle.conv1d(x1, w, bias, RELU, 1, pad, dil)
    for b in (0, 66, 131):
        e = rel_err(c_to_numpy(y[b:b + 1], BF16), ref)
        assert e <= TOL[BF16], f"batch entry {b}: error {e:.3e}"
    assert torch.equal(y.view(torch.int16), y[:1].view(torch.int16).expand(B, -1, -1))
