"""ctypes binding of libpgk: argument marshalling only.

Every step of the computation runs inside the library's HIP kernels; torch is
used for device memory and the current stream.  The names mirror the C entry
points declared in include/pgk.h.  There is no CPU fallback: if the shared
library is missing the import of a function fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

from .inputs import ACT_GELU_TANH, ACT_NONE, ACT_RELU, ACT_SILU, BF16, F32  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpgk.so")

EXPORTS = ("pgk_gemm_fused", "pgk_gemm_splitk", "pgk_gemm_fused_bt", "pgk_gemm_splitk_bt", "pgk_gemm_plan",
           "pgk_gemm_fused_workspace_bytes", "pgk_gemm_splitk_workspace_bytes", "pgk_splitk_workspace_bytes",
           "pgk_gemm_fused_static", "pgk_gemm_fused_static_max_bytes",
           "pgk_splitk_auto_splits", "pgk_reduce_max", "pgk_reduce_max_workspace_bytes", "pgk_conv1d",
           "pgk_conv1d_workspace_bytes", "pgk_conv1d_out_len", "pgk_probe_mfma", "pgk_probe_stream_read",
           "pgk_probe_gemm_phases", "pgk_probe_mfma_fed",
           "pgk_status_string", "pgk_version")

# pgk_ws_flags_t
WS_ROWSUM, WS_B_TRANSPOSED, WS_UNALIGNED = 1, 2, 4

_lib = None


class PgkError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def load_library() -> ctypes.CDLL:
    """dlopen libpgk.so (built in-tree by ``build.build_library``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2511_06345_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
    lib.pgk_gemm_fused.restype = ci
    lib.pgk_gemm_fused.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, vp, ctypes.c_size_t, vp]
    lib.pgk_gemm_fused_static.restype = ci
    lib.pgk_gemm_fused_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, vp]
    lib.pgk_gemm_fused_static_max_bytes.restype = ctypes.c_size_t
    lib.pgk_gemm_fused_static_max_bytes.argtypes = []
    lib.pgk_gemm_splitk.restype = ci
    lib.pgk_gemm_splitk.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, ci, vp,
                                    ctypes.c_size_t, vp]
    lib.pgk_gemm_fused_bt.restype = ci
    lib.pgk_gemm_fused_bt.argtypes = lib.pgk_gemm_fused.argtypes
    lib.pgk_gemm_splitk_bt.restype = ci
    lib.pgk_gemm_splitk_bt.argtypes = lib.pgk_gemm_splitk.argtypes
    lib.pgk_gemm_plan.restype = ci
    lib.pgk_gemm_plan.argtypes = [i64, i64, i64, i64, ci, ci, ctypes.POINTER(ctypes.c_int32)]
    lib.pgk_splitk_workspace_bytes.restype = ctypes.c_size_t
    lib.pgk_splitk_workspace_bytes.argtypes = [i64, i64, i64, i64, ci, ci]
    lib.pgk_gemm_splitk_workspace_bytes.restype = ctypes.c_size_t
    lib.pgk_gemm_splitk_workspace_bytes.argtypes = [i64, i64, i64, i64, ci, ci, ci]
    lib.pgk_gemm_fused_workspace_bytes.restype = ctypes.c_size_t
    lib.pgk_gemm_fused_workspace_bytes.argtypes = [i64, i64, i64, i64, ci, ci]
    lib.pgk_splitk_auto_splits.restype = ci
    lib.pgk_splitk_auto_splits.argtypes = [i64, i64, i64, i64, ci, ci]
    lib.pgk_reduce_max.restype = ci
    lib.pgk_reduce_max.argtypes = [vp, vp, vp, i64, i64, i64, ci, vp, ctypes.c_size_t, vp]
    lib.pgk_reduce_max_workspace_bytes.restype = ctypes.c_size_t
    lib.pgk_reduce_max_workspace_bytes.argtypes = [i64, i64, i64, ci]
    lib.pgk_conv1d.restype = ci
    lib.pgk_conv1d.argtypes = [vp, vp, vp, vp] + [i64] * 8 + [ci, ci, vp, ctypes.c_size_t, vp]
    lib.pgk_conv1d_workspace_bytes.restype = ctypes.c_size_t
    lib.pgk_conv1d_workspace_bytes.argtypes = [i64] * 8 + [ci]
    lib.pgk_conv1d_out_len.restype = i64
    lib.pgk_conv1d_out_len.argtypes = [i64] * 5
    lib.pgk_probe_mfma.restype = ci
    lib.pgk_probe_mfma.argtypes = [ci, ci, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.pgk_probe_mfma_fed.restype = ci
    lib.pgk_probe_mfma_fed.argtypes = [ci, ci, vp, ctypes.c_size_t, ctypes.c_size_t, ci, vp,
                                       ctypes.POINTER(ctypes.c_double), vp]
    lib.pgk_probe_gemm_phases.restype = ci
    lib.pgk_probe_gemm_phases.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, ci, ci, vp, ctypes.c_size_t,
                                          ctypes.POINTER(ctypes.c_int32), vp]
    lib.pgk_probe_stream_read.restype = ci
    lib.pgk_probe_stream_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.pgk_status_string.restype = ctypes.c_char_p
    lib.pgk_status_string.argtypes = [ci]
    lib.pgk_version.restype = ci
    lib.pgk_version.argtypes = []
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().pgk_status_string(int(status)).decode()


def version() -> int:
    return int(load_library().pgk_version())


def splitk_workspace_bytes(M: int, N: int, K: int, batch: int, dtype: int, splits: int = 0) -> int:
    """Enough for either layout of B, with or without row sums, aligned operands."""
    return int(load_library().pgk_splitk_workspace_bytes(M, N, K, batch, dtype, splits))


def gemm_splitk_workspace_bytes(M: int, N: int, K: int, batch: int, dtype: int, splits: int = 0, flags: int = 0) -> int:
    return int(load_library().pgk_gemm_splitk_workspace_bytes(M, N, K, batch, dtype, splits, flags))


def gemm_fused_workspace_bytes(M: int, N: int, K: int, batch: int, dtype: int, flags: int = 0) -> int:
    return int(load_library().pgk_gemm_fused_workspace_bytes(M, N, K, batch, dtype, flags))


def reduce_max_workspace_bytes(outer: int, red: int, inner: int, dtype: int) -> int:
    return int(load_library().pgk_reduce_max_workspace_bytes(outer, red, inner, dtype))


def splitk_auto_splits(M: int, N: int, K: int, batch: int, dtype: int, splits: int = 0) -> int:
    return int(load_library().pgk_splitk_auto_splits(M, N, K, batch, dtype, splits))


def gemm_plan(M: int, N: int, K: int, batch: int, dtype: int, b_transposed: bool = False) -> dict:
    """What the fused call runs for this shape (pgk_gemm_plan): kernel, tile, K slices, workgroups."""
    out = (ctypes.c_int32 * 6)()
    rc = load_library().pgk_gemm_plan(M, N, K, batch, dtype, int(b_transposed), out)
    if rc != 0:
        raise PgkError(rc, "pgk_gemm_plan")
    return {"matrix_core": bool(out[0]), "tile": (out[1], out[2], out[3]), "slices": out[4], "workgroups": out[5]}


def _shape(A: torch.Tensor, B: torch.Tensor, b_transposed: bool = False) -> Tuple[int, int, int, int, int]:
    if A.dim() == 2:
        A = A.unsqueeze(0)
    if B.dim() == 2:
        B = B.unsqueeze(0)
    kdim, ndim = (2, 1) if b_transposed else (1, 2)
    if A.dim() != 3 or B.dim() != 3 or A.shape[0] != B.shape[0] or A.shape[2] != B.shape[kdim]:
        raise ValueError("expected A [batch, M, K] and B [batch, K, N] (transposed: [batch, N, K])")
    if not (A.is_cuda and B.is_cuda and A.is_contiguous() and B.is_contiguous()):
        raise ValueError("A and B must be contiguous device tensors")
    if A.device != B.device:
        raise ValueError("A and B must live on the same device")
    if A.dtype == torch.float32 and B.dtype == torch.float32:
        dtype = F32
    elif A.dtype == torch.bfloat16 and B.dtype == torch.bfloat16:
        dtype = BF16
    else:
        raise TypeError("A and B must both be float32 or both bfloat16")
    batch, M, K = A.shape
    return int(batch), int(M), int(B.shape[ndim]), int(K), dtype


def _check_bias(bias: Optional[torch.Tensor], N: int, device=None) -> int:
    if bias is None:
        return 0
    if not (bias.is_cuda and bias.dtype == torch.float32 and bias.is_contiguous() and bias.numel() == N):
        raise ValueError("bias must be a contiguous float32 device tensor of N elements")
    if device is not None and bias.device != device:
        raise ValueError("bias must live on the device of the operands")
    return bias.data_ptr()


def _check_out(t: torch.Tensor, what: str, shape, dtype, device) -> torch.Tensor:
    """A caller-supplied output: the kernels write `shape` elements of `dtype` from its data
    pointer on, so anything else (a view with strides, another dtype or device, fewer
    elements) must be refused here."""
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.device != device:
        raise ValueError(f"{what} must be a tensor on {device}")
    if t.dtype != dtype:
        raise TypeError(f"{what} must have dtype {dtype}, not {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    if tuple(t.shape) != tuple(shape) and not (t.numel() == _numel(shape) and t.dim() <= len(shape)):
        raise ValueError(f"{what} must have shape {tuple(shape)}, not {tuple(t.shape)}")
    return t


def _numel(shape) -> int:
    n = 1
    for d in shape:
        n *= int(d)
    return n


def _check_workspace(ws: Optional[torch.Tensor], need: int, device) -> Tuple[Optional[int], int]:
    """(pointer or None, bytes) of a caller-supplied workspace after validation."""
    if ws is None:
        if need:
            raise ValueError(f"this call needs a workspace of {need} bytes")
        return None, 0
    if not (isinstance(ws, torch.Tensor) and ws.is_cuda and ws.device == device and ws.dtype == torch.uint8
            and ws.is_contiguous()):
        raise ValueError(f"workspace must be a contiguous uint8 tensor on {device}")
    return ws.data_ptr(), ws.numel()


class _on_stream:
    """Temporaries the binding allocates itself (outputs, workspaces) must belong, in torch's
    caching allocator, to the stream the kernels run on: allocated under that stream, a block
    freed on return is not handed out again before the queued kernels are done."""

    def __init__(self, stream):
        self.ctx = torch.cuda.stream(stream) if stream is not None else None

    def __enter__(self):
        if self.ctx is not None:
            self.ctx.__enter__()

    def __exit__(self, *exc):
        if self.ctx is not None:
            self.ctx.__exit__(*exc)


def _stream_ptr(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _ws_flags(A, B, rowsum: bool, b_transposed: bool) -> int:
    flags = (WS_ROWSUM if rowsum else 0) | (WS_B_TRANSPOSED if b_transposed else 0)
    if A.data_ptr() % 16 or B.data_ptr() % 16:
        flags |= WS_UNALIGNED
    return flags


def gemm_fused(A: torch.Tensor, B: torch.Tensor, bias: Optional[torch.Tensor], act: int,
               rowsum: bool = True, out: Optional[torch.Tensor] = None,
               rowsum_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
               stream=None, b_transposed: bool = False):
    """C = act(A @ B + bias) and (optionally) rowsum = C.sum(-1) in fp32 via pgk_gemm_fused.

    Returns (C, rowsum) with C [batch, M, N] in the dtype of A and rowsum
    [batch, M] float32 (None when ``rowsum`` is False).  Asynchronous on the
    current (or given) torch stream.  ``b_transposed``: B is [batch, N, K] and the call is
    pgk_gemm_fused_bt.  ``workspace``: a uint8 device tensor of at least
    ``gemm_fused_workspace_bytes(...)`` bytes; allocated here (torch device memory) when None
    and the problem needs one.
    """
    lib = load_library()
    batch, M, N, K, dtype = _shape(A, B, b_transposed)
    entry = lib.pgk_gemm_fused_bt if b_transposed else lib.pgk_gemm_fused
    dev = A.device
    need = gemm_fused_workspace_bytes(M, N, K, batch, dtype, _ws_flags(A, B, rowsum, b_transposed))
    with _on_stream(stream):
        if workspace is None and need:
            workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
        ws_ptr, ws_bytes = _check_workspace(workspace, need, dev)
        C = (_check_out(out, "out", (batch, M, N), A.dtype, dev) if out is not None
             else torch.empty((batch, M, N), dtype=A.dtype, device=dev))
        rs = None
        if rowsum:
            rs = (_check_out(rowsum_out, "rowsum_out", (batch, M), torch.float32, dev) if rowsum_out is not None
                  else torch.empty((batch, M), dtype=torch.float32, device=dev))
        rc = entry(A.data_ptr(), B.data_ptr(), _check_bias(bias, N, dev) or None, C.data_ptr(),
                   rs.data_ptr() if rs is not None else None,
                   M, N, K, batch, int(act), dtype, ws_ptr, ws_bytes, _stream_ptr(stream) or None)
    if rc != 0:
        raise PgkError(rc, "pgk_gemm_fused_bt" if b_transposed else "pgk_gemm_fused")
    return C, rs


def gemm_fused_static(A: torch.Tensor, B: torch.Tensor, bias: Optional[torch.Tensor], act: int,
                      out: torch.Tensor, rowsum_out: Optional[torch.Tensor] = None, stream=None):
    """pgk_gemm_fused_static: the fused call with the library's fixed workspace; nothing is
    allocated here either, so both outputs are the caller's (``rowsum_out`` None: no row sums)."""
    lib = load_library()
    batch, M, N, K, dtype = _shape(A, B)
    dev = A.device
    C = _check_out(out, "out", (batch, M, N), A.dtype, dev)
    rs = _check_out(rowsum_out, "rowsum_out", (batch, M), torch.float32, dev) if rowsum_out is not None else None
    rc = lib.pgk_gemm_fused_static(A.data_ptr(), B.data_ptr(), _check_bias(bias, N, dev) or None, C.data_ptr(),
                                   rs.data_ptr() if rs is not None else None,
                                   M, N, K, batch, int(act), dtype, _stream_ptr(stream) or None)
    if rc != 0:
        raise PgkError(rc, "pgk_gemm_fused_static")
    return C, rs


def gemm_fused_static_max_bytes() -> int:
    return int(load_library().pgk_gemm_fused_static_max_bytes())


def gemm_fused_bt(A: torch.Tensor, Bt: torch.Tensor, bias: Optional[torch.Tensor], act: int, **kw):
    """C = act(A @ Bt^T + bias) with Bt [batch, N, K] read in place (pgk_gemm_fused_bt)."""
    return gemm_fused(A, Bt, bias, act, b_transposed=True, **kw)


def gemm_splitk(A: torch.Tensor, B: torch.Tensor, bias: Optional[torch.Tensor], act: int,
                splits: int = 0, rowsum: bool = True, out: Optional[torch.Tensor] = None,
                rowsum_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                stream=None, b_transposed: bool = False):
    """Two-pass split-K variant (pgk_gemm_splitk; pgk_gemm_splitk_bt when ``b_transposed``).
    ``workspace`` is a uint8 device tensor of at least ``gemm_splitk_workspace_bytes(...)`` bytes
    (``splitk_workspace_bytes(...)`` is enough for aligned operands); allocated here when None."""
    lib = load_library()
    batch, M, N, K, dtype = _shape(A, B, b_transposed)
    entry = lib.pgk_gemm_splitk_bt if b_transposed else lib.pgk_gemm_splitk
    dev = A.device
    need = gemm_splitk_workspace_bytes(M, N, K, batch, dtype, splits, _ws_flags(A, B, rowsum, b_transposed))
    with _on_stream(stream):
        if workspace is None:
            workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=dev)
        ws_ptr, ws_bytes = _check_workspace(workspace, need, dev)
        C = (_check_out(out, "out", (batch, M, N), A.dtype, dev) if out is not None
             else torch.empty((batch, M, N), dtype=A.dtype, device=dev))
        rs = None
        if rowsum:
            rs = (_check_out(rowsum_out, "rowsum_out", (batch, M), torch.float32, dev) if rowsum_out is not None
                  else torch.empty((batch, M), dtype=torch.float32, device=dev))
        rc = entry(A.data_ptr(), B.data_ptr(), _check_bias(bias, N, dev) or None, C.data_ptr(),
                   rs.data_ptr() if rs is not None else None,
                   M, N, K, batch, int(act), dtype, int(splits), ws_ptr, ws_bytes, _stream_ptr(stream) or None)
    if rc != 0:
        raise PgkError(rc, "pgk_gemm_splitk_bt" if b_transposed else "pgk_gemm_splitk")
    return C, rs


def gemm_splitk_bt(A: torch.Tensor, Bt: torch.Tensor, bias: Optional[torch.Tensor], act: int, **kw):
    """Split-K variant with Bt [batch, N, K] read in place (pgk_gemm_splitk_bt)."""
    return gemm_splitk(A, Bt, bias, act, b_transposed=True, **kw)


def reduce_max(X: torch.Tensor, dim: int, want_idx: bool = True, out: Optional[torch.Tensor] = None,
               idx_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """Maximum of X over dimension ``dim`` and the first position attaining it
    (pgk_reduce_max).  X: contiguous float32 or bfloat16 device tensor.  Returns
    (values in the dtype of X with ``dim`` removed, int32 positions or None).  ``workspace``: uint8
    device tensor of at least ``reduce_max_workspace_bytes(...)`` bytes, allocated here when None."""
    lib = load_library()
    if not (X.is_cuda and X.is_contiguous()):
        raise ValueError("X must be a contiguous device tensor")
    if X.dtype == torch.float32:
        dtype = F32
    elif X.dtype == torch.bfloat16:
        dtype = BF16
    else:
        raise TypeError("X must be float32 or bfloat16")
    dim = dim % X.dim()
    outer = inner = 1
    for d in X.shape[:dim]:
        outer *= int(d)
    for d in X.shape[dim + 1:]:
        inner *= int(d)
    red = int(X.shape[dim])
    shape = tuple(X.shape[:dim]) + tuple(X.shape[dim + 1:])
    dev = X.device
    need = reduce_max_workspace_bytes(outer, red, inner, dtype)
    with _on_stream(stream):
        if workspace is None and need:
            workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
        ws_ptr, ws_bytes = _check_workspace(workspace, need, dev)
        vals = _check_out(out, "out", shape, X.dtype, dev) if out is not None else torch.empty(shape, dtype=X.dtype, device=dev)
        idx = None
        if want_idx:
            idx = (_check_out(idx_out, "idx_out", shape, torch.int32, dev) if idx_out is not None
                   else torch.empty(shape, dtype=torch.int32, device=dev))
        rc = lib.pgk_reduce_max(X.data_ptr(), vals.data_ptr(), idx.data_ptr() if idx is not None else None,
                                outer, red, inner, dtype, ws_ptr, ws_bytes, _stream_ptr(stream) or None)
    if rc != 0:
        raise PgkError(rc, "pgk_reduce_max")
    return vals, idx


def probe_mfma(dtype: int, random_operands: bool, iters: int, sink: torch.Tensor, stream=None) -> float:
    """Enqueues the matrix-instruction-only loop (pgk_probe_mfma); returns its flop count."""
    flops = ctypes.c_double(0.0)
    rc = load_library().pgk_probe_mfma(int(dtype), int(bool(random_operands)), int(iters), sink.data_ptr(),
                                       ctypes.byref(flops), _stream_ptr(stream) or None)
    if rc != 0:
        raise PgkError(rc, "pgk_probe_mfma")
    return float(flops.value)


def probe_mfma_fed(iters: int, clock_out: torch.Tensor, src: Optional[torch.Tensor] = None, resident_bytes: int = 0,
                   stream_every: int = 0, stream=None) -> float:
    """Enqueues the matrix-instruction loop fed from LDS (pgk_probe_mfma_fed), with the 64 KiB copies
    per iteration when `src` (contiguous bf16 device tensor, a multiple of 64 KiB) is given;
    `clock_out`: int64 device tensor of at least 3 words.  Returns the flop count of the launch."""
    if not (clock_out.is_cuda and clock_out.dtype == torch.int64 and clock_out.is_contiguous() and clock_out.numel() >= 3):
        raise ValueError("clock_out must be a contiguous int64 device tensor of at least 3 words")
    src_ptr, src_bytes = None, 0
    if src is not None:
        if not (src.is_cuda and src.dtype == torch.bfloat16 and src.is_contiguous() and src.device == clock_out.device):
            raise ValueError("src must be a contiguous bfloat16 tensor on the device of clock_out")
        src_ptr, src_bytes = src.data_ptr(), src.numel() * 2
    flops = ctypes.c_double(0.0)
    rc = load_library().pgk_probe_mfma_fed(int(src is not None), int(iters), src_ptr, src_bytes, int(resident_bytes),
                                           int(stream_every), clock_out.data_ptr(), ctypes.byref(flops),
                                           _stream_ptr(stream) or None)
    if rc != 0:
        raise PgkError(rc, "pgk_probe_mfma_fed")
    return float(flops.value)


STAMP_WORDS = 16      # uint64 per workgroup written by pgk_probe_gemm_phases


def probe_gemm_phases(A: torch.Tensor, B: torch.Tensor, bias: Optional[torch.Tensor], act: int, out: torch.Tensor,
                      stamps: torch.Tensor, rowsum_partials: Optional[torch.Tensor] = None, stream=None) -> int:
    """One launch of the timed instance of the large-tile kernel of the operands' type
    (pgk_probe_gemm_phases); `stamps` is an int64 device tensor of at least 16 words per workgroup.
    Returns the number of workgroups."""
    batch, M, N, K, dtype = _shape(A, B)
    if batch != 1:
        raise ValueError("the phase probe takes one problem (batch 1)")
    dev = A.device
    C = _check_out(out, "out", (1, M, N), A.dtype, dev)
    if not (stamps.is_cuda and stamps.dtype == torch.int64 and stamps.is_contiguous() and stamps.device == dev):
        raise ValueError("stamps must be a contiguous int64 device tensor")
    wgs = ctypes.c_int32(0)
    rc = load_library().pgk_probe_gemm_phases(
        A.data_ptr(), B.data_ptr(), _check_bias(bias, N, dev) or None, C.data_ptr(),
        rowsum_partials.data_ptr() if rowsum_partials is not None else None, M, N, K, int(act), dtype,
        stamps.data_ptr(), stamps.numel() * 8, ctypes.byref(wgs), _stream_ptr(stream) or None)
    if rc != 0:
        raise PgkError(rc, "pgk_probe_gemm_phases")
    return int(wgs.value)


def probe_stream_read(src: torch.Tensor, sink: torch.Tensor, stream=None) -> int:
    """Enqueues one streaming read of the whole of `src` (pgk_probe_stream_read); returns its bytes."""
    nbytes = src.numel() * src.element_size()
    rc = load_library().pgk_probe_stream_read(src.data_ptr(), nbytes, sink.data_ptr(), _stream_ptr(stream) or None)
    if rc != 0:
        raise PgkError(rc, "pgk_probe_stream_read")
    return nbytes


def conv1d_out_len(L: int, Kw: int, stride: int = 1, pad: int = 0, dilation: int = 1) -> int:
    return int(load_library().pgk_conv1d_out_len(L, Kw, stride, pad, dilation))


def conv1d_workspace_bytes(B: int, Cin: int, L: int, Cout: int, Kw: int, stride: int, pad: int, dilation: int,
                           dtype: int) -> int:
    return int(load_library().pgk_conv1d_workspace_bytes(B, Cin, L, Cout, Kw, stride, pad, dilation, dtype))


def conv1d(x: torch.Tensor, w: torch.Tensor, bias: Optional[torch.Tensor], act: int = ACT_NONE, stride: int = 1,
           pad: int = 0, dilation: int = 1, out: Optional[torch.Tensor] = None,
           workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """y = act(conv1d(x, w) + bias) via pgk_conv1d.  x [B, Cin, L], w [Cout, Cin, Kw]: contiguous
    float32 or bfloat16 device tensors; bias float32 [Cout] or None.  ``workspace``: uint8 device
    tensor of at least ``conv1d_workspace_bytes(...)`` bytes, allocated here when None."""
    lib = load_library()
    if x.dim() != 3 or w.dim() != 3 or x.shape[1] != w.shape[1]:
        raise ValueError("expected x [B, Cin, L] and w [Cout, Cin, Kw]")
    if not (x.is_cuda and w.is_cuda and x.is_contiguous() and w.is_contiguous() and x.device == w.device):
        raise ValueError("x and w must be contiguous tensors on one device")
    if x.dtype == torch.float32 and w.dtype == torch.float32:
        dtype = F32
    elif x.dtype == torch.bfloat16 and w.dtype == torch.bfloat16:
        dtype = BF16
    else:
        raise TypeError("x and w must both be float32 or both bfloat16")
    B, Cin, L = (int(d) for d in x.shape)
    Cout, _, Kw = (int(d) for d in w.shape)
    Lout = conv1d_out_len(L, Kw, stride, pad, dilation)
    if Lout <= 0:
        raise ValueError("the convolution has no output for these sizes")
    dev = x.device
    need = conv1d_workspace_bytes(B, Cin, L, Cout, Kw, stride, pad, dilation, dtype)
    with _on_stream(stream):
        if workspace is None and need:
            workspace = torch.empty((need,), dtype=torch.uint8, device=dev)
        ws_ptr, ws_bytes = _check_workspace(workspace, need, dev)
        y = (_check_out(out, "out", (B, Cout, Lout), x.dtype, dev) if out is not None
             else torch.empty((B, Cout, Lout), dtype=x.dtype, device=dev))
        rc = lib.pgk_conv1d(x.data_ptr(), w.data_ptr(), _check_bias(bias, Cout, dev) or None, y.data_ptr(),
                            B, Cin, L, Cout, Kw, stride, pad, dilation, int(act), dtype,
                            ws_ptr, ws_bytes, _stream_ptr(stream) or None)
    if rc != 0:
        raise PgkError(rc, "pgk_conv1d")
    return y
