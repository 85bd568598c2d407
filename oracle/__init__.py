"""CPU oracle for the fused GEMM + epilogue operator.  TEST INFRASTRUCTURE ONLY.

Thin ctypes loader around ``pgk_oracle.c`` (plain C, double precision, the
textbook definition of the operator).  Nothing here is part of the product
path: only the tests, the smoke check and the CPU-baseline leg of the
benchmark import this package, and it imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pgk_oracle.c")
_LIB = os.path.join(_HERE, "libpgk_oracle.so")

ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_SILU = 0, 1, 2, 3
F32, BF16 = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math, no FP contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_gemm_fused.restype = ctypes.c_int
        lib.oracle_gemm_fused.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_int64,
            ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_act.restype = ctypes.c_double
        lib.oracle_act.argtypes = [ctypes.c_double, ctypes.c_int]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_reduce_max.restype = ctypes.c_int
        lib.oracle_reduce_max.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                          ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_conv1d.restype = ctypes.c_int64
        lib.oracle_conv1d.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int] + \
            [ctypes.c_int64] * 8 + [ctypes.c_int, ctypes.c_void_p]
        _lib = lib
    return _lib


def act(x: float, kind: int) -> float:
    """One activation value in double (ReLU / tanh-form GELU / SiLU / identity)."""
    return float(_load().oracle_act(float(x), int(kind)))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def gemm_fused(A: np.ndarray, B: np.ndarray, bias, act_kind: int, rows=None,
               want_c: bool = True, want_rowsum: bool = True):
    """Evaluate C = act(A @ B + bias) and rowsum(C) in double.

    A: [batch, M, K] or [M, K]; B: [batch, K, N] or [K, N].  dtype float32, or
    uint16 holding bfloat16 bit patterns.  bias: float32 [N] or None.
    rows: optional 1-D int array of row indices; only those rows are evaluated.
    Returns (C, rowsum) as float64 arrays of shape [batch, R, N] and [batch, R]
    (None for a part that was not requested).
    """
    lib = _load()
    A = np.ascontiguousarray(A)
    B = np.ascontiguousarray(B)
    if A.ndim == 2:
        A = A[None]
    if B.ndim == 2:
        B = B[None]
    if A.dtype == np.float32 and B.dtype == np.float32:
        dtype = F32
    elif A.dtype == np.uint16 and B.dtype == np.uint16:
        dtype = BF16
    else:
        raise TypeError("A and B must both be float32 or both uint16 (bf16 bits)")
    batch, M, K = A.shape
    if B.shape[0] != batch or B.shape[1] != K:
        raise ValueError("shape mismatch between A and B")
    N = B.shape[2]
    bias_p = None
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if bias.shape != (N,):
            raise ValueError("bias must have shape [N]")
        bias_p = bias.ctypes.data
    rows_p, nrows, R = None, 0, M
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        rows_p, nrows, R = rows.ctypes.data, rows.size, rows.size
    C = np.empty((batch, R, N), dtype=np.float64) if want_c else None
    rs = np.empty((batch, R), dtype=np.float64) if want_rowsum else None
    rc = lib.oracle_gemm_fused(A.ctypes.data, B.ctypes.data, bias_p, M, N, K, batch,
                               int(act_kind), dtype, rows_p, nrows,
                               C.ctypes.data if want_c else None,
                               rs.ctypes.data if want_rowsum else None)
    if rc != 0:
        raise ValueError("oracle_gemm_fused rejected its arguments")
    return C, rs


def gemm_fused_bt(A: np.ndarray, Bt: np.ndarray, bias, act_kind: int, **kw):
    """The same operator with the second factor given transposed, Bt [batch, N, K] or [N, K]:
    C = act(A @ Bt^T + bias).  By definition: transpose, then the plain evaluation."""
    Bt = np.asarray(Bt)
    return gemm_fused(A, np.ascontiguousarray(np.swapaxes(Bt, -1, -2)), bias, act_kind, **kw)


def reduce_max(X: np.ndarray, dim: int, want_idx: bool = True):
    """Maximum of X over dimension `dim` and the first position attaining it.

    X: float32, or uint16 holding bfloat16 bit patterns; any number of dimensions.
    Returns (values float32 with `dim` removed, indices int32 or None).  A NaN in a
    slice gives NaN and the position of the first NaN.
    """
    lib = _load()
    X = np.ascontiguousarray(X)
    if X.dtype == np.float32:
        dtype = F32
    elif X.dtype == np.uint16:
        dtype = BF16
    else:
        raise TypeError("X must be float32 or uint16 (bf16 bits)")
    dim = dim % X.ndim
    outer = int(np.prod(X.shape[:dim], dtype=np.int64))
    red = int(X.shape[dim])
    inner = int(np.prod(X.shape[dim + 1:], dtype=np.int64))
    shape = X.shape[:dim] + X.shape[dim + 1:]
    out = np.empty(outer * inner, dtype=np.float32)
    idx = np.empty(outer * inner, dtype=np.int32) if want_idx else None
    rc = lib.oracle_reduce_max(X.ctypes.data, dtype, outer, red, inner, out.ctypes.data,
                               idx.ctypes.data if want_idx else None)
    if rc != 0:
        raise ValueError("oracle_reduce_max rejected its arguments")
    return out.reshape(shape), (idx.reshape(shape) if want_idx else None)


def conv1d_out_len(L: int, Kw: int, stride: int = 1, pad: int = 0, dilation: int = 1) -> int:
    return (L + 2 * pad - dilation * (Kw - 1) - 1) // stride + 1


def conv1d(x: np.ndarray, w: np.ndarray, bias, act_kind: int = ACT_NONE, stride: int = 1, pad: int = 0,
           dilation: int = 1) -> np.ndarray:
    """y = act(conv1d(x, w) + bias) in double.  x [B, Cin, L], w [Cout, Cin, Kw]: float32, or
    uint16 holding bfloat16 bits; bias float32 [Cout] or None.  Cross-correlation with zero
    padding, as in deep-learning frameworks.  Returns float64 [B, Cout, Lout]."""
    lib = _load()
    x, w = np.ascontiguousarray(x), np.ascontiguousarray(w)
    if x.dtype == np.float32 and w.dtype == np.float32:
        dtype = F32
    elif x.dtype == np.uint16 and w.dtype == np.uint16:
        dtype = BF16
    else:
        raise TypeError("x and w must both be float32 or both uint16 (bf16 bits)")
    if x.ndim != 3 or w.ndim != 3 or x.shape[1] != w.shape[1]:
        raise ValueError("expected x [B, Cin, L] and w [Cout, Cin, Kw]")
    B, Cin, L = x.shape
    Cout, _, Kw = w.shape
    bias_p = None
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.float32)
        if bias.shape != (Cout,):
            raise ValueError("bias must have shape [Cout]")
        bias_p = bias.ctypes.data
    Lout = conv1d_out_len(L, Kw, stride, pad, dilation)
    if Lout <= 0:
        raise ValueError("empty output")
    y = np.empty((B, Cout, Lout), dtype=np.float64)
    rc = lib.oracle_conv1d(x.ctypes.data, w.ctypes.data, bias_p, dtype, B, Cin, L, Cout, Kw,
                           stride, pad, dilation, int(act_kind), y.ctypes.data)
    if rc != Lout:
        raise ValueError("oracle_conv1d rejected its arguments")
    return y
