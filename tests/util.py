"""Helpers shared by the GPU parity tests (no arithmetic of the operator itself)."""
import numpy as np

from paper_2511_06345_amd import inputs as gen

TOL = {gen.F32: 1e-4, gen.BF16: 2e-2}   # max relative error bar per element type


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_i |g_i - r_i| / max(|r_i|, RMS(r)): relative error with the tensor's RMS as
    the floor of the denominator, so that entries near zero (ReLU zeros, activation
    tails, sums that cancel) are judged against the scale of the tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return float(np.max(np.abs(got - ref)))
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))


def to_device(arr: np.ndarray, dtype: int):
    import torch
    if dtype == gen.BF16:
        return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(arr).cuda()


def c_to_numpy(C, dtype: int) -> np.ndarray:
    """Device C -> float64 numpy (bf16 widened exactly)."""
    import torch
    if dtype == gen.BF16:
        bits = C.view(torch.int16).cpu().numpy().view(np.uint16)
        return gen.bf16_bits_to_f32(bits).astype(np.float64)
    return C.cpu().numpy().astype(np.float64)


def sample_rows(M: int, tile: int, n_random: int, seed: int) -> np.ndarray:
    """Rows on both sides of every tile boundary plus seeded random rows."""
    rows = {0, M - 1}
    for t in range(tile, M, tile):
        rows.update((t - 1, t))
    if len(rows) > 4 * n_random:           # many tiles: keep a seeded subset of the boundary rows
        rng = np.random.default_rng(seed + 1)
        rows = set(rng.choice(sorted(rows), size=4 * n_random, replace=False).tolist()) | {0, M - 1}
    rng = np.random.default_rng(seed)
    rows.update(rng.integers(0, M, n_random).tolist())
    return np.array(sorted(rows), dtype=np.int64)


def strict_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """Unjudged companion of rel_err: plain max |g - r| / |r| over the entries with |r| >= RMS(r)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    big = np.abs(ref) >= rms
    if not big.any():
        return 0.0
    return float(np.max(np.abs(got[big] - ref[big]) / np.abs(ref[big])))


def abs_inputs(A: np.ndarray, B: np.ndarray, bias, dtype: int):
    """|A|, |B|, |bias| in the storage format of the inputs (bf16 bit patterns: sign bit cleared)."""
    if dtype == gen.BF16:
        a, b = A & np.uint16(0x7FFF), B & np.uint16(0x7FFF)
    else:
        a, b = np.abs(A), np.abs(B)
    return a, b, (np.abs(bias) if bias is not None else None)
