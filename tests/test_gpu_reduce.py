"""GPU parity of the max reduction: the HIP kernels (through the C ABI) against the CPU
oracle, bit for bit -- a maximum is exact and positions are integers, so values must have
identical bit patterns (NaN where the oracle has NaN) and positions must be equal."""
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


def values_to_numpy(v, dtype):
    import torch
    if dtype == BF16:
        return gen.bf16_bits_to_f32(v.view(torch.int16).cpu().numpy().view(np.uint16))
    return v.cpu().numpy()


def same_bits(got, ref, what):
    got, ref = np.ascontiguousarray(got, dtype=np.float32), np.ascontiguousarray(ref, dtype=np.float32)
    assert got.shape == ref.shape, what
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan), f"{what}: NaN placement"
    assert np.array_equal(got.view(np.uint32)[~nan], ref.view(np.uint32)[~nan]), f"{what}: value bits"


def make(dtype, shape, seed, kind):
    n = int(np.prod(shape))
    if kind == "normal":
        x = gen.normal(gen.tensor_seed(96, 1, seed), n, 1.0)
    elif kind == "ties":
        x = gen.small_ints(gen.tensor_seed(96, 2, seed), n, -2, 2)
    else:   # specials sprinkled over normal data: signed zeros, infinities, a few NaNs
        x = gen.normal(gen.tensor_seed(96, 3, seed), n, 1.0)
        pick = gen.uniform(gen.tensor_seed(96, 4, seed), n, 0.0, 1.0)
        x[pick < 0.30] = 0.0
        x[pick < 0.15] = -0.0
        x[(pick > 0.40) & (pick < 0.41)] = np.inf
        x[(pick > 0.50) & (pick < 0.52)] = -np.inf
        x[(pick > 0.60) & (pick < 0.6005)] = np.nan
    x = x.reshape(shape)
    return gen.f32_to_bf16_bits(x) if dtype == BF16 else x


def run_and_compare(pgk, oracle, X, dtype, dim, what, misalign=False):
    import torch
    if misalign:    # same numbers at an address that is not a multiple of 16
        esz = 2 if dtype == BF16 else 4
        flat = to_device(np.concatenate([np.zeros(1, dtype=X.dtype), X.reshape(-1)]), dtype)
        dX = flat[1:].view(X.shape)
        assert dX.data_ptr() % 16 == esz and dX.is_contiguous()
    else:
        dX = to_device(X, dtype)
    ref_v, ref_i = oracle.reduce_max(X, dim)
    v, i = pgk.reduce_max(dX, dim)
    torch.cuda.synchronize()
    same_bits(values_to_numpy(v, dtype), ref_v, what)
    assert np.array_equal(i.cpu().numpy(), ref_i), f"{what}: positions"
    v2, none = pgk.reduce_max(dX, dim, want_idx=False)
    torch.cuda.synchronize()
    assert none is None
    same_bits(values_to_numpy(v2, dtype), ref_v, what + " (values only)")


# [outer, red, inner] views reached through (shape, dim).  Contiguous reduced dimension:
# short rows (one wave each), long rows (a workgroup each), few long rows (segments + second
# pass), lengths that are not multiples of the 16-byte chunk (scalar fallback).  Strided
# reduced dimension: wide and narrow inner extents, ragged inner tails, few outputs with a
# long reduced dimension (segments), odd inner extents (scalar fallback).
SHAPES = [
    ((1, 1), 1), ((5, 1), 0), ((3, 7), 1), ((3, 7), 0), ((300, 520), 1), ((1000, 64), 1),
    ((37, 4096), 1), ((6, 40000), 1), ((3, 1 << 20), 1), ((2, 1000003), 1), ((700, 2052), 1),
    ((4, 9, 512), 1), ((3, 1000, 1032), 1), ((2, 5000, 72), 1), ((1, 30000, 8), 1), ((5, 77, 333), 1),
    ((4096, 40), 0), ((70000, 6), 0), ((9, 4, 5, 6), 2), ((2, 3, 4, 2048), 1),
    # very short rows (several rows per wave: 1 ... 32 lanes each, vector and scalar loads)
    ((1000, 8), 1), ((5000, 32), 1), ((777, 100), 1), ((333, 512), 1), ((2000, 3), 1), ((401, 128), 1), ((300, 129), 1),
    ((65, 1024), 1), ((100, 33), 1),
    # small inner extents (one wave per outer index sweeping the flattened block; with and without segments)
    ((300, 50, 3), 1), ((7, 1000, 5), 1), ((2, 100000, 2), 1), ((5, 77, 33), 1), ((64, 64, 64), 1), ((9, 4, 5, 6), 1),
    ((3, 40000, 40), 1), ((1000, 7, 5), 1), ((50000, 2), 0), ((1, 3, 64), 1),
    # blocks of red x inner <= 128 elements (several outer indices per workgroup)
    ((100000, 7, 5), 1), ((1001, 2, 64), 1), ((37, 64, 2), 1), ((5, 1, 100), 1), ((3000, 3, 3), 1), ((2, 43, 3), 0),
]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("kind", ["normal", "ties", "specials"])
def test_shapes_and_splits(pgk, oracle, dtype, kind):
    for n, (shape, dim) in enumerate(SHAPES):
        X = make(dtype, shape, 100 * n + dim, kind)
        run_and_compare(pgk, oracle, X, dtype, dim, f"{shape} dim {dim} {kind}")


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_misaligned_base_address(pgk, oracle, dtype):
    for n, (shape, dim) in enumerate([((300, 520), 1), ((3, 1 << 18), 1), ((3, 1000, 1032), 1), ((4096, 40), 0)]):
        X = make(dtype, shape, 7 + n, "ties")
        run_and_compare(pgk, oracle, X, dtype, dim, f"misaligned {shape} dim {dim}", misalign=True)


def test_planted_maximum_is_found_everywhere(pgk, oracle):
    """One large value moved through every position of a row and of a column: each lane,
    sweep, wave and segment boundary is hit."""
    import torch
    red = 3000
    X = np.zeros((red, red), dtype=np.float32)
    X[np.arange(red), np.arange(red)] = 7.0            # row r has its maximum at column r
    dX = torch.from_numpy(X).cuda()
    for dim in (0, 1):
        v, i = pgk.reduce_max(dX, dim)
        torch.cuda.synchronize()
        assert np.all(v.cpu().numpy() == 7.0) and np.array_equal(i.cpu().numpy(), np.arange(red, dtype=np.int32))
    long_row = np.zeros((1, 1 << 22), dtype=np.float32)
    for at in (0, 1, 1023, 1024, 4095, 4096, (1 << 21) - 1, 1 << 21, (1 << 22) - 1):
        long_row[:] = 0.0
        long_row[0, at] = 1.0
        v, i = pgk.reduce_max(torch.from_numpy(long_row).cuda(), 1)
        torch.cuda.synchronize()
        assert v.item() == 1.0 and i.item() == at


def test_is_deterministic(pgk):
    import torch
    X = to_device(make(F32, (3, 1 << 20), 5, "ties"), F32)
    a = pgk.reduce_max(X, 1)
    b = pgk.reduce_max(X, 1)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


@pytest.mark.parametrize("name", sorted(gen.REDUCE_WORKLOADS))
def test_reduce_workloads_full_size(pgk, oracle, name):
    """The benchmark's reduction workloads at full size, every output compared."""
    w = gen.REDUCE_WORKLOADS[name]
    X = gen.make_reduce_input(w)
    run_and_compare(pgk, oracle, X, w.dtype, w.dim, name)


@pytest.mark.parametrize("dim", [1, 2])
def test_tensor_larger_than_4_gib(pgk, oracle, dim):
    """[72, 4096, 4100] fp32 = 4.8 GB, a seeded [4096, 4100] block repeated along the first
    dimension: element offsets of the later entries exceed 32 bits; every entry must reduce
    like the block does (strided and contiguous dimension; rows of 4100 are not tile multiples)."""
    import torch
    block = make(F32, (4096, 4100), 31, "ties")
    ref_v, ref_i = oracle.reduce_max(block, dim - 1)
    X = to_device(block, F32)[None].expand(72, -1, -1).contiguous()
    assert X.numel() * 4 > (1 << 32)
    v, i = pgk.reduce_max(X, dim)
    torch.cuda.synchronize()
    for o in (0, 1, 35, 71):
        same_bits(v[o].cpu().numpy(), ref_v, f"entry {o} dim {dim}")
        assert np.array_equal(i[o].cpu().numpy(), ref_i), f"positions of entry {o} dim {dim}"
    assert torch.equal(v, v[:1].expand_as(v)) and torch.equal(i, i[:1].expand_as(i))
