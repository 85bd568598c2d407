"""Pins for the max-reduction oracle (CPU only): it is checked against numpy's max /
argmax (a library routine), hand cases, the defining properties by brute force on tiny
inputs, and the special values, so that a wrong stride, a `>=` for `>`, or a dropped
dimension fails at least one of them."""
import itertools

import numpy as np
import pytest

from paper_2511_06345_amd import inputs as gen


def _f32(a):
    return np.asarray(a, dtype=np.float32)


def test_hand_case(oracle):
    X = _f32([[1, 5, 3], [4, 2, 6]])
    v, i = oracle.reduce_max(X, 0)
    assert v.tolist() == [4, 5, 6] and i.tolist() == [1, 0, 1]
    v, i = oracle.reduce_max(X, 1)
    assert v.tolist() == [5, 6] and i.tolist() == [1, 2]
    X3 = _f32(np.arange(24).reshape(2, 3, 4))
    v, i = oracle.reduce_max(X3, 1)
    assert np.array_equal(v, X3[:, 2, :]) and np.all(i == 2)
    v, i = oracle.reduce_max(-X3, 1)
    assert np.array_equal(v, -X3[:, 0, :]) and np.all(i == 0)


@pytest.mark.parametrize("shape", [(7,), (3, 5), (4, 6, 5), (2, 3, 4, 5), (1, 9, 1), (5, 1, 7), (33, 17, 65)])
def test_agrees_with_numpy_max_and_argmax(oracle, shape):
    n = int(np.prod(shape))
    X = gen.normal(gen.tensor_seed(95, 1, n), n, 1.0).reshape(shape)
    for dim in range(len(shape)):
        v, i = oracle.reduce_max(X, dim)
        assert np.array_equal(v, X.max(axis=dim))
        assert np.array_equal(i, X.argmax(axis=dim).astype(np.int32))
        v2, none = oracle.reduce_max(X, dim - len(shape), want_idx=False)
        assert none is None and np.array_equal(v2, v)


@pytest.mark.parametrize("shape", [(6, 40, 9), (3, 200), (50, 3, 2)])
def test_ties_go_to_the_first_position(oracle, shape):
    n = int(np.prod(shape))
    X = gen.small_ints(gen.tensor_seed(95, 2, n), n, -1, 1).astype(np.float32).reshape(shape)   # three values: many ties
    for dim in range(len(shape)):
        v, i = oracle.reduce_max(X, dim)
        assert np.array_equal(v, X.max(axis=dim))
        assert np.array_equal(i, X.argmax(axis=dim).astype(np.int32))     # numpy: first occurrence


def test_defining_properties_by_brute_force(oracle):
    X = gen.small_ints(gen.tensor_seed(95, 3, 0), 3 * 4 * 5, -3, 3).astype(np.float32).reshape(3, 4, 5)
    for dim in range(3):
        v, i = oracle.reduce_max(X, dim)
        Xm = np.moveaxis(X, dim, 0)
        for pos in itertools.product(*[range(s) for s in v.shape]):
            col = [float(Xm[(r,) + pos]) for r in range(Xm.shape[0])]
            assert all(c <= v[pos] for c in col)              # not exceeded
            assert col[i[pos]] == v[pos]                      # attained where it says
            assert all(c < v[pos] for c in col[:i[pos]])      # nothing equal before it


def test_value_is_invariant_under_permutation_of_the_reduced_axis(oracle):
    X = gen.normal(gen.tensor_seed(95, 4, 0), 5 * 31 * 6, 2.0).reshape(5, 31, 6)
    perm = np.argsort(gen.uniform(gen.tensor_seed(95, 5, 0), 31, 0.0, 1.0))
    v, i = oracle.reduce_max(X, 1)
    vp, ip = oracle.reduce_max(X[:, perm, :], 1)
    assert np.array_equal(v, vp)
    assert np.array_equal(perm[ip], i)        # no ties in continuous data: same element found


def test_reduced_length_one_is_the_identity(oracle):
    X = gen.normal(gen.tensor_seed(95, 6, 0), 12, 1.0).reshape(3, 1, 4)
    v, i = oracle.reduce_max(X, 1)
    assert np.array_equal(v, X[:, 0, :]) and np.all(i == 0)


def test_dimension_split_is_consistent(oracle):
    """Reducing dimension d equals reducing the last dimension after moving d there:
    two different (outer, reduced, inner) decompositions of the same numbers."""
    X = gen.normal(gen.tensor_seed(95, 7, 0), 4 * 5 * 6 * 3, 1.0).reshape(4, 5, 6, 3)
    for dim in range(4):
        v, i = oracle.reduce_max(X, dim)
        vm, im = oracle.reduce_max(np.ascontiguousarray(np.moveaxis(X, dim, -1)), -1)
        assert np.array_equal(v, vm) and np.array_equal(i, im)


def test_signed_zeros_compare_equal_and_the_first_wins(oracle):
    v, i = oracle.reduce_max(_f32([-0.0, 0.0, -0.0]), 0)
    assert i == 0 and np.signbit(v)
    v, i = oracle.reduce_max(_f32([0.0, -0.0]), 0)
    assert i == 0 and not np.signbit(v)
    v, i = oracle.reduce_max(_f32([-1.0, -0.0, 0.0]), 0)
    assert i == 1 and np.signbit(v) and v == 0


def test_nan_and_infinity(oracle):
    nan, inf = np.nan, np.inf
    v, i = oracle.reduce_max(_f32([1, nan, 5, nan]), 0)
    assert np.isnan(v) and i == 1
    v, i = oracle.reduce_max(_f32([nan, 7]), 0)
    assert np.isnan(v) and i == 0
    v, i = oracle.reduce_max(_f32([-inf, -inf]), 0)
    assert v == -inf and i == 0
    v, i = oracle.reduce_max(_f32([1, inf, inf, 2]), 0)
    assert v == inf and i == 1
    X = _f32([[1, nan], [3, 4], [nan, 9]])
    v, i = oracle.reduce_max(X, 0)
    assert np.isnan(v).all() and i.tolist() == [2, 0]
    v, i = oracle.reduce_max(X, 1)
    assert np.isnan(v[0]) and v[1] == 4 and np.isnan(v[2]) and i.tolist() == [1, 1, 0]


def test_bf16_bit_patterns_are_widened_exactly(oracle):
    vals = gen.normal(gen.tensor_seed(95, 8, 0), 6 * 50, 3.0).reshape(6, 50)
    bits = gen.f32_to_bf16_bits(vals)
    wide = gen.bf16_bits_to_f32(bits)
    for dim in (0, 1):
        v, i = oracle.reduce_max(bits, dim)
        assert np.array_equal(v, wide.max(axis=dim))
        assert np.array_equal(i, wide.argmax(axis=dim).astype(np.int32))
    # every finite bf16 pattern in one row: the largest finite value is 0x7F7F
    allbits = np.array([b for b in range(65536) if (b & 0x7F80) != 0x7F80], dtype=np.uint16)
    v, i = oracle.reduce_max(allbits, 0)
    assert allbits[i] == 0x7F7F and v == gen.bf16_bits_to_f32(np.array([0x7F7F], dtype=np.uint16))[0]


def test_rejects_bad_arguments(oracle):
    with pytest.raises(TypeError):
        oracle.reduce_max(np.zeros((2, 2), dtype=np.float64), 0)
    with pytest.raises(ValueError):
        oracle.reduce_max(np.zeros((2, 0), dtype=np.float32), 1)
