"""Pins for the conv1d oracle (CPU only): numpy's correlate per channel pair (a library
routine), the width-one kernel against a matrix product, unit-impulse kernels, the all-ones
closed form, linearity, shift equivariance and integer exactness -- chosen so that a flipped
kernel (convolution instead of correlation), a wrong padding offset, swapped stride and
dilation, or a dropped channel fails at least one."""
import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen


def rnd(shape, seed, scale=1.0):
    n = int(np.prod(shape))
    return gen.normal(gen.tensor_seed(97, 1, seed), n, scale).reshape(shape)


def numpy_conv1d(x, w, bias, stride, pad, dilation):
    """Independent route: zero-pad, dilate the kernel with zeros, numpy.correlate per
    (output channel, input channel), subsample by the stride."""
    B, Cin, L = x.shape
    Cout, _, Kw = w.shape
    xp = np.zeros((B, Cin, L + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + L] = x
    wd = np.zeros((Cout, Cin, dilation * (Kw - 1) + 1), dtype=np.float64)
    wd[:, :, ::dilation] = w
    full = xp.shape[2] - wd.shape[2] + 1
    y = np.zeros((B, Cout, full), dtype=np.float64)
    for b in range(B):
        for co in range(Cout):
            for ci in range(Cin):
                y[b, co] += np.correlate(xp[b, ci], wd[co, ci], mode="valid")
            if bias is not None:
                y[b, co] += float(bias[co])
    return y[:, :, ::stride]


def test_hand_case(oracle):
    x = np.array([[[1, 2, 3, 4]]], dtype=np.float32)
    w = np.array([[[1, 0, -1]]], dtype=np.float32)          # y[l] = x[l] - x[l+2]: correlation, not convolution
    assert oracle.conv1d(x, w, None).tolist() == [[[-2.0, -2.0]]]
    assert oracle.conv1d(x, w, None, pad=1).tolist() == [[[-2.0, -2.0, -2.0, 3.0]]]
    assert oracle.conv1d(x, w, np.array([10], dtype=np.float32), pad=1, stride=2).tolist() == [[[8.0, 8.0]]]
    assert oracle.conv1d(x, np.array([[[1, 1]]], dtype=np.float32), None, dilation=3).tolist() == [[[5.0]]]
    assert oracle.conv1d_out_len(4, 3) == 2 and oracle.conv1d_out_len(4, 3, pad=1, stride=2) == 2


@pytest.mark.parametrize("cfg", [  # B, Cin, L, Cout, Kw, stride, pad, dilation
    (1, 1, 9, 1, 3, 1, 0, 1), (2, 3, 17, 4, 3, 1, 1, 1), (2, 3, 17, 4, 5, 2, 2, 1), (1, 2, 30, 3, 4, 3, 5, 2),
    (3, 5, 40, 2, 7, 1, 3, 3), (1, 4, 13, 6, 1, 2, 0, 1), (2, 2, 21, 2, 2, 1, 4, 5)])
def test_agrees_with_numpy_correlate(oracle, cfg):
    B, Cin, L, Cout, Kw, stride, pad, dilation = cfg
    x, w = rnd((B, Cin, L), 1 + L), rnd((Cout, Cin, Kw), 2 + Kw)
    bias = rnd((Cout,), 3)
    got = oracle.conv1d(x, w, bias, stride=stride, pad=pad, dilation=dilation)
    ref = numpy_conv1d(x, w, bias, stride, pad, dilation)
    assert got.shape == ref.shape == (B, Cout, oracle.conv1d_out_len(L, Kw, stride, pad, dilation))
    assert np.max(np.abs(got - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_width_one_kernel_is_a_matrix_product(oracle):
    x, w = rnd((3, 6, 25), 11), rnd((5, 6, 1), 12)
    bias = rnd((5,), 13)
    got = oracle.conv1d(x, w, bias, gen.ACT_SILU)
    c, _ = oracle.gemm_fused(np.broadcast_to(w[:, :, 0], (3, 5, 6)).copy(), x, None, gen.ACT_NONE, want_rowsum=False)
    ref = c + bias[None, :, None].astype(np.float64)
    ref = ref / (1.0 + np.exp(-ref))
    assert np.max(np.abs(got - ref)) <= 1e-12


def test_unit_impulse_kernels_shift_the_input(oracle):
    x = rnd((2, 1, 20), 21)
    for k in range(4):
        w = np.zeros((1, 1, 4), dtype=np.float32)
        w[0, 0, k] = 1.0
        y = oracle.conv1d(x, w, None, pad=3)                 # y[l] = x[l + k - 3], zero outside
        ref = np.zeros((2, 1, 23))
        for l in range(23):
            if 0 <= l + k - 3 < 20:
                ref[:, 0, l] = x[:, 0, l + k - 3]
        assert np.array_equal(y, ref)


def test_all_ones_counts_the_taps_inside_the_input(oracle):
    B, Cin, L, Cout, Kw, pad, dilation = 1, 3, 12, 2, 5, 4, 2
    y = oracle.conv1d(np.ones((B, Cin, L), np.float32), np.ones((Cout, Cin, Kw), np.float32), None, pad=pad, dilation=dilation)
    for l in range(y.shape[2]):
        taps = sum(1 for k in range(Kw) if 0 <= l + k * dilation - pad < L)
        assert np.all(y[:, :, l] == Cin * taps)


def test_linearity_and_shift_equivariance(oracle):
    x1, x2, w = rnd((2, 3, 31), 31), rnd((2, 3, 31), 32), rnd((4, 3, 3), 33)
    y = oracle.conv1d(x1 + x2, w, None, pad=1)
    assert np.max(np.abs(y - oracle.conv1d(x1, w, None, pad=1) - oracle.conv1d(x2, w, None, pad=1))) <= 1e-6
    assert np.array_equal(oracle.conv1d(4 * x1, w, None), 4 * oracle.conv1d(x1, w, None))     # exact power of two
    shifted = np.zeros_like(x1)
    shifted[:, :, 5:] = x1[:, :, :-5]
    a, b = oracle.conv1d(x1, w, None), oracle.conv1d(shifted, w, None)
    assert np.array_equal(a[:, :, :-5], b[:, :, 5:])                                          # no padding: interior shifts along


def test_integer_inputs_match_int64(oracle):
    B, Cin, L, Cout, Kw = 2, 7, 50, 3, 4
    x = gen.small_ints(gen.tensor_seed(97, 5, 0), B * Cin * L).reshape(B, Cin, L)
    w = gen.small_ints(gen.tensor_seed(97, 6, 0), Cout * Cin * Kw).reshape(Cout, Cin, Kw)
    for dt in ("f32", "bf16"):
        xa, wa = (x, w) if dt == "f32" else (gen.f32_to_bf16_bits(x), gen.f32_to_bf16_bits(w))
        y = oracle.conv1d(xa, wa, None, stride=2, pad=2)
        xi = np.pad(x.astype(np.int64), ((0, 0), (0, 0), (2, 2)))
        ref = np.zeros(y.shape, dtype=np.int64)
        for l in range(y.shape[2]):
            ref[:, :, l] = np.einsum("bck,ock->bo", xi[:, :, 2 * l:2 * l + Kw], w.astype(np.int64))
        assert np.array_equal(y, ref.astype(np.float64))


def test_rejects_bad_arguments(oracle):
    x, w = rnd((1, 2, 5), 41), rnd((1, 2, 3), 42)
    with pytest.raises(ValueError):
        oracle.conv1d(x, w, None, dilation=3)        # kernel span 7 exceeds the input: empty output
    with pytest.raises(ValueError):
        oracle.conv1d(x, rnd((1, 3, 3), 43), None)   # channel mismatch
    with pytest.raises(TypeError):
        oracle.conv1d(x.astype(np.float64), w, None)
