"""Pins for the CPU oracle (oracle/pgk_oracle.c).

The paper (PRAGMA, Sections 1 and 4.2) only names the operator families; the
operator is the textbook GEMM + bias + activation + row sum, so every pin below
is a mathematical fact about that definition, chosen so that a dropped term, a
wrong sign or index, or a transposed operand fails at least one of them.
None of these tests touches a GPU.
"""
import math
import os

import numpy as np
import pytest
import torch

from paper_2511_06345_amd import inputs as gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

NONE, RELU, GELU, SILU = 0, 1, 2, 3


def f32(x):
    return np.asarray(x, dtype=np.float32)


# ----------------------------------------------------------------- hand cases
def test_hand_2x2(oracle):
    A = f32([[1, 2], [3, 4]])
    B = f32([[5, 6], [7, 8]])
    C, rs = oracle.gemm_fused(A, B, None, NONE)
    assert C[0].tolist() == [[19.0, 22.0], [43.0, 50.0]]
    assert rs[0].tolist() == [41.0, 93.0]
    C, rs = oracle.gemm_fused(A, B, f32([-20, -45]), RELU)
    assert C[0].tolist() == [[0.0, 0.0], [23.0, 5.0]]
    assert rs[0].tolist() == [0.0, 28.0]


def test_hand_non_square_detects_transposition(oracle):
    # 2x3 times 3x2 with asymmetric entries: A.B != (B^T.A^T) unless indices are right
    A = f32([[1, 2, 3], [4, 5, 6]])
    B = f32([[1, 0], [0, 2], [3, 1]])
    C, rs = oracle.gemm_fused(A, B, f32([10, 100]), NONE)
    assert C[0].tolist() == [[20.0, 107.0], [32.0, 116.0]]
    assert rs[0].tolist() == [127.0, 148.0]


def test_hand_transposed_second_factor(oracle):
    # the same product with the second factor handed over as its transpose [N][K]
    A = f32([[1, 2, 3], [4, 5, 6]])
    Bt = f32([[1, 0, 3], [0, 2, 1]])
    C, rs = oracle.gemm_fused_bt(A, Bt, f32([10, 100]), NONE)
    assert C[0].tolist() == [[20.0, 107.0], [32.0, 116.0]]
    assert rs[0].tolist() == [127.0, 148.0]
    # a linear layer by hand: y = x W^T + b with W [out=3][in=2]
    x = f32([[1, -1]])
    W = f32([[2, 3], [5, 7], [-1, 4]])
    C, _ = oracle.gemm_fused_bt(x, W, f32([0.5, 0, 1]), RELU)
    assert C[0].tolist() == [[0.0, 0.0, 0.0]]
    C, _ = oracle.gemm_fused_bt(x, W, f32([1.5, 0, 6]), NONE)
    assert C[0].tolist() == [[0.5, -2.0, 1.0]]


@pytest.mark.parametrize("seed,shape", [(10, (33, 17, 65, 2)), (11, (8, 128, 40, 1))])
def test_transposed_against_numpy_float64(oracle, seed, shape):
    M, N, K, batch = shape
    rng = np.random.default_rng(seed)
    A = rng.uniform(-1, 1, (batch, M, K)).astype(np.float32)
    Bt = rng.uniform(-1, 1, (batch, N, K)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    ref = np.einsum("bmk,bnk->bmn", A.astype(np.float64), Bt.astype(np.float64)) + bias.astype(np.float64)
    C, rs = oracle.gemm_fused_bt(A, Bt, bias, NONE)
    assert np.max(np.abs(C - ref)) <= 1e-12 * max(np.sqrt(np.mean(ref ** 2)), 1.0)
    assert np.max(np.abs(rs - ref.sum(axis=2))) <= 1e-11 * np.sqrt(N) * max(np.sqrt(np.mean(ref ** 2)), 1.0)


def test_degenerate_shapes(oracle):
    C, rs = oracle.gemm_fused(f32([[3]]), f32([[-2]]), f32([1]), NONE)       # 1x1x1
    assert C.ravel().tolist() == [-5.0] and rs.ravel().tolist() == [-5.0]
    a = f32([[2], [3], [5]])                                                 # K = 1: outer product
    b = f32([[1, -1, 4, 0]])
    C, rs = oracle.gemm_fused(a, b, None, NONE)
    assert np.array_equal(C[0], np.outer([2, 3, 5], [1, -1, 4, 0]).astype(np.float64))
    row = f32([[1, 2, 3, 4]])                                                # M = 1, N = 1: dot product
    col = f32([[1], [10], [100], [1000]])
    C, rs = oracle.gemm_fused(row, col, None, NONE)
    assert C.ravel().tolist() == [4321.0]


def test_batch_is_independent(oracle):
    rng = np.random.default_rng(1)
    A = rng.integers(-3, 4, (3, 5, 7)).astype(np.float32)
    B = rng.integers(-3, 4, (3, 7, 4)).astype(np.float32)
    bias = rng.integers(-3, 4, 4).astype(np.float32)
    C, rs = oracle.gemm_fused(A, B, bias, RELU)
    for b in range(3):
        Cb, rsb = oracle.gemm_fused(A[b], B[b], bias, RELU)
        assert np.array_equal(C[b], Cb[0]) and np.array_equal(rs[b], rsb[0])


# -------------------------------------------------- identity and permutation
@pytest.mark.parametrize("act", [NONE, RELU, GELU, SILU])
def test_identity_and_permutation(oracle, act):
    rng = np.random.default_rng(2)
    n = 17
    B = rng.standard_normal((n, 23)).astype(np.float32)
    bias = rng.standard_normal(23).astype(np.float32)
    expect = np.array([[oracle.act(float(B[i, j]) + float(bias[j]), act) for j in range(23)]
                       for i in range(n)])
    C, _ = oracle.gemm_fused(np.eye(n, dtype=np.float32), B, bias, act)
    assert np.array_equal(C[0], expect)
    perm = rng.permutation(n)
    P = np.zeros((n, n), dtype=np.float32)
    P[np.arange(n), perm] = 1.0
    C, _ = oracle.gemm_fused(P, B, bias, act)
    assert np.array_equal(C[0], expect[perm])


# ------------------------------------------------------------ closed forms
@pytest.mark.parametrize("M,N,K", [(3, 5, 7), (4, 256, 65536), (2, 3, 1)])
def test_all_ones(oracle, M, N, K):
    C, rs = oracle.gemm_fused(np.ones((M, K), np.float32), np.ones((K, N), np.float32), None, NONE)
    assert np.all(C == float(K)) and np.all(rs == float(N) * float(K))


def test_rowsum_closed_form(oracle):
    """rowsum equals C.1, and for the identity activation equals A.(B.1) + sum(bias)."""
    rng = np.random.default_rng(3)
    A = rng.standard_normal((2, 9, 31)).astype(np.float32)
    B = rng.standard_normal((2, 31, 13)).astype(np.float32)
    bias = rng.standard_normal(13).astype(np.float32)
    for act in (NONE, RELU, GELU, SILU):
        C, rs = oracle.gemm_fused(A, B, bias, act)
        np.testing.assert_allclose(rs, C.sum(axis=2), rtol=1e-13, atol=1e-13)
    C, rs = oracle.gemm_fused(A, B, bias, NONE)
    matvec = np.einsum("bik,bk->bi", A.astype(np.float64), B.astype(np.float64).sum(axis=2))
    np.testing.assert_allclose(rs, matvec + bias.astype(np.float64).sum(), rtol=1e-12, atol=1e-12)


def test_linearity_and_transpose(oracle):
    rng = np.random.default_rng(4)
    A1 = rng.standard_normal((6, 11)).astype(np.float32)
    A2 = rng.standard_normal((6, 11)).astype(np.float32)
    B1 = rng.standard_normal((11, 8)).astype(np.float32)
    B2 = rng.standard_normal((11, 8)).astype(np.float32)
    g = lambda a, b: oracle.gemm_fused(a, b, None, NONE)[0][0]
    # powers of two scale exactly
    assert np.array_equal(g(f32(4.0) * A1, B1), 4.0 * g(A1, B1))
    assert np.array_equal(g(A1, f32(0.25) * B1), 0.25 * g(A1, B1))
    # additivity (A1 + A2 is rounded to fp32 first, so use exactly representable sums)
    Ai = rng.integers(-8, 9, (6, 11)).astype(np.float32)
    Aj = rng.integers(-8, 9, (6, 11)).astype(np.float32)
    np.testing.assert_allclose(g(Ai + Aj, B1), g(Ai, B1) + g(Aj, B1), rtol=1e-13, atol=1e-13)
    Bi = rng.integers(-8, 9, (11, 8)).astype(np.float32)
    Bj = rng.integers(-8, 9, (11, 8)).astype(np.float32)
    np.testing.assert_allclose(g(A1, Bi + Bj), g(A1, Bi) + g(A1, Bj), rtol=1e-13, atol=1e-13)
    # (A B)^T = B^T A^T
    np.testing.assert_allclose(g(A1, B2).T, g(np.ascontiguousarray(B2.T), np.ascontiguousarray(A1.T)),
                               rtol=1e-13, atol=1e-13)
    # bias is added once per column, to every row
    bias = rng.standard_normal(8).astype(np.float32)
    Cb = oracle.gemm_fused(A2, B2, bias, NONE)[0][0]
    np.testing.assert_allclose(Cb - g(A2, B2), np.broadcast_to(bias.astype(np.float64), (6, 8)),
                               rtol=0, atol=1e-13)


# ------------------------------------------------------------ integer exact
@pytest.mark.parametrize("dtype", [gen.F32, gen.BF16])
@pytest.mark.parametrize("shape", [(5, 7, 33, 2), (64, 48, 1000, 1), (3, 2, 40000, 1)])
def test_integer_exact_vs_int64(oracle, dtype, shape):
    M, N, K, batch = shape
    A, B = gen.make_int_inputs(dtype, M, N, K, batch, seed=77)
    Af = gen.bf16_bits_to_f32(A) if dtype == gen.BF16 else A
    Bf = gen.bf16_bits_to_f32(B) if dtype == gen.BF16 else B
    ref = np.matmul(Af.astype(np.int64), Bf.astype(np.int64))
    bias = np.arange(N, dtype=np.float32) - 3
    C, rs = oracle.gemm_fused(A, B, bias, NONE)
    assert np.array_equal(C, (ref + bias.astype(np.int64)).astype(np.float64))
    assert np.array_equal(rs, (ref + bias.astype(np.int64)).sum(axis=2).astype(np.float64))
    C, _ = oracle.gemm_fused(A, B, bias, RELU)
    assert np.array_equal(C, np.maximum(ref + bias.astype(np.int64), 0).astype(np.float64))


def test_bf16_widening_is_exact(oracle):
    # every finite bf16 bit pattern times 1 comes back as the same value
    bits = np.arange(0, 1 << 16, dtype=np.uint32)
    finite = ((bits >> 7) & 0xFF) != 0xFF
    bits = bits[finite].astype(np.uint16)
    n = bits.size
    one = gen.f32_to_bf16_bits(np.ones((1, 1), np.float32))
    C, _ = oracle.gemm_fused(bits.reshape(n, 1), one, None, NONE)
    assert np.array_equal(C[0, :, 0], gen.bf16_bits_to_f32(bits).astype(np.float64))


# ----------------------------------------------------- float64 library routine
@pytest.mark.parametrize("seed,shape", [(0, (64, 64, 64, 1)), (1, (127, 61, 257, 2)), (2, (256, 256, 256, 1)),
                                        (3, (1, 509, 13, 3)), (4, (300, 7, 512, 1))])
def test_against_numpy_float64(oracle, seed, shape):
    M, N, K, batch = shape
    rng = np.random.default_rng(seed)
    A = rng.uniform(-1, 1, (batch, M, K)).astype(np.float32)
    B = rng.uniform(-1, 1, (batch, K, N)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    x = np.matmul(A.astype(np.float64), B.astype(np.float64)) + bias.astype(np.float64)
    xt = torch.from_numpy(x)
    refs = {
        NONE: x,
        RELU: torch.relu(xt).numpy(),
        GELU: torch.nn.functional.gelu(xt, approximate="tanh").numpy(),
        SILU: torch.nn.functional.silu(xt).numpy(),
    }
    for act, ref in refs.items():
        C, rs = oracle.gemm_fused(A, B, bias, act)
        scale = np.sqrt(np.mean(ref ** 2))
        assert np.max(np.abs(C - ref)) <= 1e-12 * max(scale, 1.0)
        assert np.max(np.abs(rs - ref.sum(axis=2))) <= 1e-11 * max(scale, 1.0) * np.sqrt(N)


def test_row_subset_matches_full(oracle):
    rng = np.random.default_rng(5)
    A = rng.standard_normal((2, 40, 19)).astype(np.float32)
    B = rng.standard_normal((2, 19, 6)).astype(np.float32)
    bias = rng.standard_normal(6).astype(np.float32)
    C, rs = oracle.gemm_fused(A, B, bias, SILU)
    rows = np.array([39, 0, 7, 7, 21])
    Cs, rss = oracle.gemm_fused(A, B, bias, SILU, rows=rows)
    assert np.array_equal(Cs, C[:, rows]) and np.array_equal(rss, rs[:, rows])


# ------------------------------------------------------------- activations
def test_activation_closed_forms(oracle):
    ln3, ln2 = math.log(3.0), math.log(2.0)
    # logistic sigma(ln 3) = 3/4, sigma(ln 2) = 2/3, sigma(-ln 3) = 1/4
    assert oracle.act(ln3, SILU) == pytest.approx(0.75 * ln3, rel=1e-15)
    assert oracle.act(ln2, SILU) == pytest.approx(2.0 / 3.0 * ln2, rel=1e-15)
    assert oracle.act(-ln3, SILU) == pytest.approx(-0.25 * ln3, rel=1e-15)
    # tanh(ln(3)/2) = 1/2 : solve sqrt(2/pi) (x + 0.044715 x^3) = ln(3)/2 by bisection,
    # then GELU_tanh(x) = 0.75 x
    target = ln3 / 2.0
    lo, hi = 0.0, 2.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if math.sqrt(2.0 / math.pi) * (mid + 0.044715 * mid ** 3) < target:
            lo = mid
        else:
            hi = mid
    x = 0.5 * (lo + hi)
    assert oracle.act(x, GELU) == pytest.approx(0.75 * x, rel=1e-13)
    assert oracle.act(-x, GELU) == pytest.approx(-0.25 * x, rel=1e-13)
    for act in (NONE, RELU, GELU, SILU):
        assert oracle.act(0.0, act) == 0.0
    assert math.copysign(1.0, oracle.act(-0.0, RELU)) == 1.0      # ReLU(-0) = +0
    assert oracle.act(-2.5, RELU) == 0.0 and oracle.act(2.5, RELU) == 2.5
    assert oracle.act(-2.5, NONE) == -2.5


@pytest.mark.parametrize("act", [RELU, GELU, SILU])
def test_activation_odd_part_and_limits(oracle, act):
    # f(x) - f(-x) = x for ReLU, tanh-GELU and SiLU alike
    for x in [1e-3, 0.1, 0.5, 1.0, 2.0, 3.3, 7.0, 20.0]:
        assert oracle.act(x, act) - oracle.act(-x, act) == pytest.approx(x, rel=1e-14, abs=1e-16)
    assert oracle.act(50.0, act) == pytest.approx(50.0, rel=1e-15)
    assert abs(oracle.act(-50.0, act)) < 1e-15
    assert oracle.act(-3.0, act) <= 0.0 and oracle.act(3.0, act) > 2.8


def test_gelu_tanh_close_to_exact_gelu(oracle):
    """The tanh form approximates x.Phi(x); a wrong constant breaks the known error bound."""
    worst = 0.0
    for i in range(-800, 801):
        x = i / 100.0
        exact = 0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0)))
        worst = max(worst, abs(oracle.act(x, GELU) - exact))
    assert 1e-4 < worst < 1e-3


def test_activation_golden_table(oracle):
    """Values tabulated independently (double precision, standard published forms)."""
    name_to_act = {"gelu_tanh": GELU, "silu": SILU, "relu": RELU}
    n = 0
    with open(os.path.join(GOLDEN, "activation_values.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            name, x, y = line.split()
            # abs term: the literal 0.5 x (1 + tanh u) form loses the far negative tail
            # (|value| < 1e-15 |x|) to cancellation in double; irrelevant at the 1e-4 parity bar
            assert oracle.act(float(x), name_to_act[name]) == pytest.approx(float(y), rel=2e-15, abs=2e-15)
            n += 1
    assert n >= 20


# ------------------------------------------------------------ input generator
def test_generator_is_reproducible_and_distributed():
    a = gen.uniform(123, 100000, -1.0, 1.0)
    b = gen.uniform(123, 100000, -1.0, 1.0)
    assert np.array_equal(a, b) and a.dtype == np.float32
    assert -1.0 <= a.min() and a.max() <= 1.0 and abs(a.mean()) < 0.01
    assert abs(a.std() - 1.0 / math.sqrt(3.0)) < 0.01
    z = gen.normal(321, 200000, 0.1)
    assert abs(z.mean()) < 1e-3 and abs(z.std() - 0.1) < 1e-3
    # counter-based: a later window equals the tail of a longer draw
    assert np.array_equal(gen.splitmix64(9, 5, 10), gen.splitmix64(9, 0, 15)[5:])
    # first output of SplitMix64 seeded with 0 (published reference value)
    assert int(gen.splitmix64(0, 0, 1)[0]) == 0xE220A8397B1DCDAF
    ints = gen.small_ints(5, 10000)
    assert set(np.unique(ints).tolist()) == {-2.0, -1.0, 0.0, 1.0, 2.0}


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8], np.float32)
    bits = gen.f32_to_bf16_bits(x)
    back = gen.bf16_bits_to_f32(bits)
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(back, t)
    # ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even mantissa (1.0)
    assert back[5] == 1.0 and back[6] == np.float32(1.0 + 2 ** -6)


def test_workload_table_matches_recipe():
    w = gen.WORKLOADS
    assert (w["c1"].M, w["c1"].N, w["c1"].K, w["c1"].batch) == (256, 256, 256, 1)
    assert (w["c3"].M, w["c3"].dtype, w["c3"].act, w["c3"].rowsum) == (8192, gen.BF16, gen.ACT_SILU, False)
    assert (w["c4"].M, w["c4"].N, w["c4"].K) == (16384, 1024, 4096) and w["c4"].rowsum
    assert (w["c5"].K, w["c5"].batch, w["c5"].call) == (65536, 16, "splitk")
    assert w["c3"].flops == 2.0 * 8192 ** 3
    A, B, bias = gen.make_inputs(w["c1"])
    assert A.shape == (1, 256, 256) and B.shape == (1, 256, 256) and bias.shape == (256,)
    A4, B4, bias4 = gen.make_inputs(w["c4"], shape=(64, 32, 128, 1))
    assert A4.dtype == np.uint16 and abs(gen.bf16_bits_to_f32(B4).std() - 1.0 / 64.0) < 2e-3
    assert gen.make_inputs(w["c5"], shape=(8, 8, 64, 2))[2] is None
