"""libpgk: fused GEMM + bias/activation/row-sum kernels and a max reduction for AMD MI355X (gfx950).

``inputs`` (seeded synthetic workloads) imports nothing but numpy; the GPU
binding is loaded lazily on first use of ``gemm_fused`` / ``gemm_splitk`` / ``reduce_max``.
"""
from . import inputs  # noqa: F401

_LAZY = {"gemm_fused", "gemm_splitk", "gemm_fused_bt", "gemm_splitk_bt", "reduce_max", "conv1d", "splitk_workspace_bytes", "splitk_auto_splits",
         "gemm_fused_workspace_bytes", "gemm_splitk_workspace_bytes", "reduce_max_workspace_bytes",
         "status_string", "version", "load_library", "PgkError"}


def __getattr__(name):
    if name in _LAZY:
        import importlib
        return getattr(importlib.import_module(__name__ + ".binding"), name)
    raise AttributeError(name)
