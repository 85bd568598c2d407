"""The C-ABI library without a GPU: it loads, exports every declared symbol, and
rejects bad arguments on the host before any device work (no compute calls here)."""
import ctypes

import numpy as np
import os
import re

import pytest

from paper_2511_06345_amd import binding
from paper_2511_06345_amd import inputs as gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, INVALID, UNSUPPORTED, WORKSPACE, HIP = 0, -1, -2, -3, -4


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_06345_amd.build import build_library
        build_library()
    return binding.load_library()


def test_exports_match_header(lib):
    text = open(os.path.join(ROOT, "include", "pgk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(pgk_[a-z_0-9]+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_library_is_built_from_the_sources_as_they_stand(lib):
    """The GPU tests, smoke() and bench.py load the library that is there: a library older than
    the sources would be tested in place of the code."""
    from paper_2511_06345_amd import build
    assert os.path.exists(build.BUILT_FROM), "libpgk.so carries no record of its sources: rebuild it"
    assert open(build.BUILT_FROM).read().strip() == build.source_hash(), \
        "csrc/ has changed since libpgk.so was built: run `python -m paper_2511_06345_amd.build`"


def test_version_and_status_strings(lib):
    assert binding.version() == 200
    seen = set()
    for code in (OK, INVALID, UNSUPPORTED, WORKSPACE, HIP, 12345):
        s = binding.status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert binding.status_string(OK) == "PGK_OK"


def _fused(lib, A=0x1000, B=0x2000, bias=None, C=0x3000, rs=None, M=4, N=4, K=4, batch=1, act=0, dtype=0, ws=None,
           ws_bytes=0, bt=False):
    fn = lib.pgk_gemm_fused_bt if bt else lib.pgk_gemm_fused
    return fn(A, B, bias, C, rs, M, N, K, batch, act, dtype, ws, ws_bytes, None)


def test_fused_rejects_bad_arguments_on_the_host(lib):
    # the pointers are never dereferenced: validation happens before any HIP call
    assert _fused(lib, A=None) == INVALID
    assert _fused(lib, B=None) == INVALID
    assert _fused(lib, C=None) == INVALID
    for bad in ({"M": 0}, {"N": -1}, {"K": 0}, {"batch": 0}, {"act": 4}, {"act": -1}, {"dtype": 2}, {"dtype": -1}):
        assert _fused(lib, **bad) == INVALID, bad
    assert _fused(lib, M=1 << 31) == UNSUPPORTED
    assert _fused(lib, M=(1 << 31) - 1, N=(1 << 31) - 1, K=8, batch=2) == UNSUPPORTED


def test_fused_workspace_is_the_callers(lib):
    """The library owns no device memory: whatever a call needs beyond inputs and outputs comes
    from the workspace argument, the query says how much, and a call without it is refused on
    the host (nothing is launched; the pointers here are never dereferenced)."""
    F32, BF16 = gen.F32, gen.BF16
    q = binding.gemm_fused_workspace_bytes
    RS, BT, UN = binding.WS_ROWSUM, binding.WS_B_TRANSPOSED, binding.WS_UNALIGNED
    # the large workloads without row sums: nothing
    assert q(8192, 8192, 8192, 1, BF16) == 0 and q(4096, 4096, 4096, 1, F32) == 0
    assert q(8192, 8192, 8192, 1, BF16, BT) == 0
    # row sums over four tile columns of 256: one fp32 partial per row and tile column
    assert q(16384, 1024, 4096, 1, BF16, RS) == 4 * 16384 * 4
    assert q(16384, 1024, 4096, 1, BF16) == 0
    # the small fp32 workload: eight tile columns of 32 (the K-splitting tile of latency-bound problems)
    assert q(256, 256, 256, 1, F32, RS) == 8 * 256 * 4
    # one tile column: the kernel's row sums are final
    assert q(65536, 128, 1024, 1, BF16, RS) == 0
    # few tiles and a long K: the partial products of the automatic split (8 slices here)
    assert binding.gemm_plan(1024, 1024, 8192, 1, BF16)["slices"] == 8
    assert q(1024, 1024, 8192, 1, BF16) == 8 * 1024 * 1024 * 4
    assert q(256, 256, 65536, 16, F32, RS) == binding.splitk_workspace_bytes(256, 256, 65536, 16, F32, 0)
    # bf16 rows off the 4-byte grid: zero-padded copies of both operands (K 515 -> 520, N 251 -> 256)
    r256 = lambda n: -(-n // 256) * 256          # every piece starts on a multiple of 256 bytes
    assert q(130, 251, 515, 1, BF16) == r256(130 * 520 * 2) + r256(520 * 256 * 2)
    assert q(130, 251, 515, 1, BF16, BT) == r256(130 * 520 * 2) + r256(251 * 520 * 2)
    # misaligned operands of a tile-friendly problem: copies of both, rows as they are
    assert q(128, 256, 192, 2, F32, UN) == 2 * 128 * 192 * 4 + 2 * 192 * 256 * 4
    assert q(128, 256, 192, 2, F32) == 0
    # too small to be worth a copy: the bounds-checked kernel, row-sum partials per 64-column tile
    assert q(5, 7, 33, 2, BF16, RS | UN) == 0
    assert q(33, 130, 17, 1, BF16, RS) == r256(3 * 33 * 4)
    # invalid queries
    assert q(0, 4, 4, 1, F32) == 0 and q(4, 4, 4, 1, 7) == 0 and q(4, 4, 4, 1, F32, 8) == 0
    # the calls check what they are given
    need = q(16384, 1024, 4096, 1, BF16, RS)
    big = dict(M=16384, N=1024, K=4096, dtype=BF16)
    assert _fused(lib, rs=0x5000, **big) == WORKSPACE
    assert _fused(lib, rs=0x5000, ws=0x10000, ws_bytes=need - 1, **big) == WORKSPACE
    assert _fused(lib, rs=0x5000, ws=0x10004, ws_bytes=need + 16, **big) == WORKSPACE      # misaligned
    assert _fused(lib, A=0x1002, M=128, N=256, K=192, dtype=BF16) == WORKSPACE            # a misaligned operand is copied
    assert _fused(lib, M=1024, N=1024, K=8192, dtype=BF16) == WORKSPACE                    # automatic split
    assert _fused(lib, M=1024, N=1024, K=8192, dtype=BF16, bt=True) == WORKSPACE


def _splitk(lib, ws=0x4000, ws_bytes=1 << 30, splits=0, **kw):
    a = dict(A=0x1000, B=0x2000, bias=None, C=0x3000, rs=None, M=4, N=4, K=64, batch=1, act=0, dtype=0)
    a.update(kw)
    return lib.pgk_gemm_splitk(a["A"], a["B"], a["bias"], a["C"], a["rs"], a["M"], a["N"], a["K"], a["batch"],
                               a["act"], a["dtype"], splits, ws, ws_bytes, None)


def test_splitk_rejects_bad_arguments_on_the_host(lib):
    assert _splitk(lib, A=None) == INVALID
    assert _splitk(lib, K=0) == INVALID
    assert _splitk(lib, splits=-1) == INVALID
    assert _splitk(lib, splits=65, K=64) == INVALID            # more splits than K
    assert _splitk(lib, ws=None) == WORKSPACE
    assert _splitk(lib, ws_bytes=15) == WORKSPACE
    assert _splitk(lib, ws=0x4004) == WORKSPACE                # misaligned
    need = binding.splitk_workspace_bytes(4, 4, 64, 1, gen.F32, 2)
    assert _splitk(lib, splits=2, ws_bytes=need - 1) == WORKSPACE
    # the exact query never asks for more than the covering one (aligned operands) ...
    for shape, dt in (((4, 4, 64, 1), gen.F32), ((20, 2056, 512, 1), gen.BF16), ((130, 251, 515, 2), gen.BF16),
                      ((16384, 16, 4096, 1), gen.BF16), ((256, 256, 65536, 16), gen.F32)):
        cover = binding.splitk_workspace_bytes(*shape, dt, 0)
        for flags in range(4):
            assert 0 < binding.gemm_splitk_workspace_bytes(*shape, dt, 0, flags) <= cover, (shape, flags)
    # ... a skinny output's second pass keeps per-segment row sums after the partial products
    s = binding.splitk_auto_splits(20, 2056, 512, 1, gen.BF16, 0)
    assert binding.gemm_splitk_workspace_bytes(20, 2056, 512, 1, gen.BF16, 0, 0) == -(-s * 20 * 2056 * 4 // 256) * 256
    assert binding.gemm_splitk_workspace_bytes(20, 2056, 512, 1, gen.BF16, 0, binding.WS_ROWSUM) > \
        binding.gemm_splitk_workspace_bytes(20, 2056, 512, 1, gen.BF16, 0, 0)
    # ... and misaligned operands are copied into it
    assert binding.gemm_splitk_workspace_bytes(128, 128, 1024, 1, gen.F32, 2, binding.WS_UNALIGNED) == \
        2 * 128 * 128 * 4 + 2 * 128 * 1024 * 4


def test_split_plan_arithmetic(lib):
    F32, BF16 = gen.F32, gen.BF16
    # the batched tiny-output / huge-K workload: 4 tiles x 16 problems -> 8 splits fill 2 x 256 CUs
    assert binding.splitk_auto_splits(256, 256, 65536, 16, F32, 0) == 8
    assert binding.splitk_workspace_bytes(256, 256, 65536, 16, F32, 0) == 16 * 8 * 256 * 256 * 4
    assert binding.splitk_workspace_bytes(256, 256, 65536, 16, F32, 4) == 16 * 4 * 256 * 256 * 4
    # K = 100 fp32: 4 K-steps of 32; 3 splits -> 2 steps per slice -> only 2 non-empty slices
    assert binding.splitk_auto_splits(8, 8, 100, 1, F32, 3) == 2
    # never more slices than K steps; bf16 K step is 64
    assert binding.splitk_auto_splits(8, 8, 100, 1, BF16, 2) == 2
    assert binding.splitk_auto_splits(8, 8, 64, 1, BF16, 5) == 1
    # a grid that already fills the chip is not split
    assert binding.splitk_auto_splits(8192, 8192, 8192, 1, BF16, 0) == 1
    # auto choice is capped
    assert 1 <= binding.splitk_auto_splits(64, 64, 1 << 20, 1, F32, 0) <= 32
    # invalid queries
    assert binding.splitk_auto_splits(0, 8, 8, 1, F32, 0) == 0
    assert binding.splitk_workspace_bytes(8, 8, 8, 1, 7, 0) == 0
    assert binding.splitk_workspace_bytes(8, 8, 8, 1, F32, 9) == 0


def test_tile_table_and_split_rule(lib):
    """pgk_gemm_plan: the host's choice of kernel, tile and K slices, pinned on the five
    workloads and on the shapes each rule was measured on."""
    F32, BF16 = gen.F32, gen.BF16
    plan = binding.gemm_plan

    def expect(shape, dtype, tile, slices, wgs, matrix_core=True, bt=False):
        got = plan(*shape, dtype, b_transposed=bt)
        assert got == {"matrix_core": matrix_core, "tile": tile, "slices": slices, "workgroups": wgs}, (shape, dtype, got)

    # the five workloads (c5 through the fused call: same plan as the split call's automatic one)
    expect((256, 256, 256, 1), F32, (32, 32, 32), 1, 64)
    expect((4096, 4096, 4096, 1), F32, (128, 128, 32), 1, 1024)
    expect((8192, 8192, 8192, 1), BF16, (256, 256, 64), 1, 1024)
    expect((16384, 1024, 4096, 1), BF16, (256, 256, 64), 1, 256)
    expect((256, 256, 65536, 16), F32, (128, 128, 32), 8, 512)
    assert lib.pgk_splitk_auto_splits(256, 256, 65536, 16, F32, 0) == 8
    # latency-bound fp32 problems (at most 64 tiles of 64 x 64, K below 32 K tiles, plain B, K and N
    # multiples of 4): 32 x 32 tiles whose waves split K; otherwise the small tile as before
    expect((128, 128, 64, 1), F32, (32, 32, 32), 1, 16)
    expect((100, 36, 64, 2), F32, (32, 32, 32), 1, 16)
    expect((512, 512, 992, 1), F32, (32, 32, 32), 1, 256)
    expect((512, 512, 1024, 1), F32, (64, 64, 32), 2, 128)              # 32 K tiles: two passes
    expect((256, 256, 256, 1), F32, (64, 64, 32), 1, 16, bt=True)
    expect((256, 256, 32, 1), F32, (64, 64, 32), 1, 16)                 # a single K step: nothing to split
    expect((256, 258, 256, 1), F32, (64, 64, 32), 1, 20)                # N off the 16-byte grid
    expect((576, 512, 256, 1), F32, (64, 64, 32), 1, 72)                # more than 64 tiles of 64 x 64
    expect((256, 256, 256, 1), BF16, (128, 128, 64), 1, 4)
    # last tile column / row at most half full: half tiles (bf16, either layout of B)
    expect((65536, 128, 1024, 1), BF16, (256, 128, 64), 1, 256)
    expect((128, 65536, 1024, 1), BF16, (128, 256, 64), 1, 256)
    expect((65536, 128, 1024, 1), BF16, (256, 128, 64), 1, 256, bt=True)
    expect((65536, 384, 512, 1), BF16, (256, 256, 64), 1, 512)           # a quarter of padding: large tile stays
    expect((65536, 128, 1024, 1), F32, (128, 128, 32), 1, 512)
    # three quarters of a large tile empty, or a grid of few large tiles: small tile
    expect((64, 65536, 1024, 1), BF16, (128, 128, 64), 1, 512)
    expect((1024, 1024, 1024, 1), BF16, (128, 128, 64), 1, 64)
    expect((2048, 2048, 2048, 1), BF16, (128, 128, 64), 1, 256)
    # bf16 grids of at most half the CUs' worth of large tiles: one round of half (from 96 large
    # tiles and 16 K tiles on) or small tiles; one large tile more: the large tile, in one piece
    expect((2560, 3072, 4096, 1), BF16, (256, 128, 64), 1, 10 * 24)
    expect((2048, 4096, 8192, 1), BF16, (256, 128, 64), 1, 8 * 32)
    expect((2560, 3072, 512, 1), BF16, (128, 128, 64), 1, 20 * 24)
    expect((2304, 2560, 4096, 1), BF16, (128, 128, 64), 1, 18 * 20)
    expect((2816, 3072, 4096, 1), BF16, (256, 256, 64), 1, 11 * 12)
    expect((3072, 3584, 16384, 1), BF16, (256, 256, 64), 1, 12 * 14)
    expect((3584, 3584, 512, 1), BF16, (256, 256, 64), 1, 14 * 14)
    # a large-tile grid that ends in a poorly filled round, K from 1024 on: the shape the round model prefers
    expect((4097, 4096, 4096, 1), BF16, (128, 128, 64), 1, 33 * 32)
    expect((4608, 4608, 4096, 1), BF16, (256, 128, 64), 1, 18 * 36)
    expect((4097, 4096, 4096, 1), F32, (64, 64, 32), 1, 65 * 64)
    expect((3072, 3072, 4096, 1), F32, (64, 64, 32), 1, 48 * 48)
    expect((5000, 4096, 4096, 1), F32, (128, 128, 32), 1, 40 * 32)
    expect((4352, 4352, 512, 1), BF16, (256, 256, 64), 1, 17 * 17)
    # few tiles and a long K: slices of at least 16 K tiles, the fewest that give 512 workgroups
    expect((32, 8192, 8192, 1), BF16, (32, 128, 64), 8, 512)
    expect((48, 8192, 8192, 1), BF16, (128, 128, 64), 8, 512)
    expect((1024, 1024, 8192, 1), BF16, (128, 128, 64), 8, 512)
    expect((256, 256, 65536, 1), BF16, (128, 128, 64), 32, 128)
    expect((256, 256, 1024, 1), BF16, (128, 128, 64), 1, 4)                 # 16 K tiles: not worth a second pass
    # only the small-tile grid fills the chip: split from 512 K tiles on
    expect((2048, 2048, 16384, 1), BF16, (128, 128, 64), 1, 256)
    expect((2048, 2048, 65536, 1), BF16, (256, 256, 64), 4, 256)          # (one round of large tiles)
    # K or N off the 16-byte grid: read in place, or the plan of the zero-padded copies (bf16, odd)
    expect((4096, 4096, 4098, 1), F32, (128, 128, 32), 1, 1024)
    expect((4096, 4100, 4096, 1), BF16, (128, 128, 64), 1, 32 * 33)       # (17 tile columns of 256: poorly filled last round)
    expect((4096, 4101, 4096, 1), BF16, (128, 128, 64), 1, 32 * 33)
    expect((4096, 4100, 4096, 1), F32, (64, 64, 32), 1, 64 * 65)
    expect((4096, 4101, 512, 1), BF16, (256, 256, 64), 1, 16 * 17)
    # at most 32 rows or columns: the skinny tiles (flat 32 x 128, narrow 128 x 32), K in slices
    expect((8, 4096, 4096, 1), BF16, (32, 128, 64), 4, 128)
    expect((1, 4096, 4096, 1), F32, (32, 128, 32), 8, 256)
    expect((16384, 16, 16384, 1), BF16, (128, 32, 64), 4, 512)         # (a plain B of 16 columns is transposed first)
    expect((16384, 16, 16384, 1), F32, (128, 32, 32), 4, 512, bt=True)
    expect((100000, 8, 8, 1), F32, (128, 32, 32), 1, 782)
    expect((12, 12, 100000, 1), BF16, (32, 128, 64), 32, 32)           # a tiny output with a long K as well
    # an output below 16 x 16, or too little work to copy operands for: bounds-checked kernel
    expect((12, 12, 1000, 1), BF16, (64, 64, 16), 1, 1, matrix_core=False)
    expect((2, 300, 5, 1), BF16, (64, 64, 16), 1, 5, matrix_core=False)
    expect((5, 7, 33, 2), F32, (64, 64, 16), 1, 2, matrix_core=False)
    # ragged everything on the matrix cores
    expect((3000, 5000, 4104, 1), BF16, (256, 256, 64), 1, 12 * 20)
    # invalid sizes
    out = (ctypes.c_int32 * 6)()
    assert lib.pgk_gemm_plan(0, 4, 4, 1, F32, 0, out) == -1
    assert lib.pgk_gemm_plan(4, 4, 4, 1, 7, 0, out) == -1
    assert lib.pgk_gemm_plan(4, 4, 4, 1, F32, 0, None) == -1
    assert lib.pgk_gemm_plan(1 << 31, 4, 4, 1, F32, 0, out) == -2


def test_reduce_max_rejects_bad_arguments_on_the_host(lib):
    def call(X=0x1000, out=0x2000, idx=None, outer=2, red=3, inner=4, dtype=0, ws=None, ws_bytes=0):
        return lib.pgk_reduce_max(X, out, idx, outer, red, inner, dtype, ws, ws_bytes, None)
    assert call(X=None) == INVALID
    assert call(out=None) == INVALID
    for bad in ({"outer": 0}, {"red": 0}, {"inner": -3}, {"dtype": 2}):
        assert call(**bad) == INVALID, bad
    assert call(red=1 << 31) == UNSUPPORTED
    assert call(outer=1 << 40, inner=1 << 40) == UNSUPPORTED
    # few outputs, a long reduced range: two passes, the segment results in the caller's workspace
    q = binding.reduce_max_workspace_bytes
    assert q(100000, 8, 1, gen.F32) == 0 and q(2, 3, 4, gen.F32) == 0 and q(64, 4096, 1024, gen.F32) > 0
    need = q(16, 1 << 24, 1, gen.F32)
    assert need > 0 and need % 8 == 0
    assert call(outer=16, red=1 << 24, inner=1) == WORKSPACE
    assert call(outer=16, red=1 << 24, inner=1, ws=0x8000, ws_bytes=need - 8) == WORKSPACE
    assert call(outer=16, red=1 << 24, inner=1, ws=0x8002, ws_bytes=need) == WORKSPACE
    assert q(0, 3, 4, gen.F32) == 0 and q(2, 3, 4, 5) == 0


def test_conv1d_host_arithmetic_and_validation(lib):
    F32, BF16 = gen.F32, gen.BF16
    assert binding.conv1d_out_len(4, 3) == 2 and binding.conv1d_out_len(4, 3, 2, 1, 1) == 2
    assert binding.conv1d_out_len(5, 3, 1, 0, 3) == 0 and binding.conv1d_out_len(0, 3) == 0
    # matrix-core path: regrouped weights + zero-padded strips for the first and the last tile
    # column (64-column tiles on this small grid, halo 2, rounded up to 16 bytes: 68 columns)
    need = binding.conv1d_workspace_bytes(2, 64, 1000, 64, 3, 1, 1, 1, F32)
    assert need == 64 * 64 * 3 * 4 + 2 * (2 * 64) * 68 * 4
    # (32 output channels: the flat tile, 128 columns wide)
    assert binding.conv1d_workspace_bytes(2, 64, 1000, 32, 3, 1, 1, 1, F32) == 32 * 64 * 3 * 4 + 2 * (2 * 64) * 132 * 4
    # padding wider than a tile: a padded copy of the whole input instead (rows of 1000 + 2 * 101, rounded up)
    need = binding.conv1d_workspace_bytes(2, 64, 1000, 64, 3, 1, 101, 1, F32)
    assert need == 64 * 64 * 3 * 4 + 2 * 64 * 1204 * 4
    # no padding and aligned rows: only the weights
    assert binding.conv1d_workspace_bytes(2, 64, 1024, 32, 3, 1, 0, 2, F32) == 32 * 64 * 3 * 4
    # stride 2: one copy of the input per phase (rows of 500 outputs + 1 tap offset + 1, rounded up to 504)
    assert binding.conv1d_workspace_bytes(2, 64, 1000, 32, 3, 2, 1, 1, F32) == 32 * 64 * 3 * 4 + 2 * (2 * 64) * 504 * 4
    # 48 channels: copy and weights padded to 64 channels (rows of 1000 + 2 + 1, rounded up to 1004)
    assert binding.conv1d_workspace_bytes(2, 48, 1000, 32, 3, 1, 1, 1, F32) == 32 * 64 * 3 * 4 + (2 * 64) * 1004 * 4
    assert binding.conv1d_workspace_bytes(2, 64, 1000, 32, 3, 1, 2, 2, BF16) > 0
    # bf16 with odd dilation: a second copy shifted by one element for the taps at odd offsets (rows of 1008)
    assert binding.conv1d_workspace_bytes(2, 64, 1000, 32, 3, 1, 1, 1, BF16) == 32 * 64 * 3 * 2 + 2 * (2 * 64) * 1008 * 2
    # an output length that is not a multiple of 16 bytes (1001): a padded copy whose rows hold the
    # last chunk's columns and the halo (1004 + 2, rounded up to 1008)
    assert binding.conv1d_workspace_bytes(2, 64, 1001, 32, 3, 1, 1, 1, F32) == 32 * 64 * 3 * 4 + 2 * 64 * 1008 * 4
    # three channels (padding them to a K tile would multiply the work), fewer than 16 outputs
    # per row, more than 32 taps at stride 2: in place, no workspace
    assert binding.conv1d_workspace_bytes(2, 3, 1000, 32, 3, 1, 1, 1, F32) == 0
    assert binding.conv1d_workspace_bytes(2, 64, 1000, 8, 3, 1, 1, 1, F32) > 0     # (8 output channels: the flat tile)
    assert binding.conv1d_workspace_bytes(2, 64, 15, 32, 3, 1, 1, 1, F32) == 0      # 15 outputs per row
    assert binding.conv1d_workspace_bytes(2, 64, 1000, 32, 33, 2, 16, 1, F32) == 0

    def call(x=0x1000, w=0x2000, y=0x3000, B=1, Cin=4, L=16, Cout=4, Kw=3, stride=1, pad=0, dil=1, act=0, dtype=0,
             ws=None, ws_bytes=0):
        return lib.pgk_conv1d(x, w, None, y, B, Cin, L, Cout, Kw, stride, pad, dil, act, dtype, ws, ws_bytes, None)
    assert call(x=None) == INVALID and call(w=None) == INVALID and call(y=None) == INVALID
    for bad in ({"B": 0}, {"Cin": 0}, {"Kw": 0}, {"stride": 0}, {"pad": -1}, {"dil": 0}, {"act": 9}, {"dtype": 3},
                {"L": 2, "Kw": 3}):
        assert call(**bad) == INVALID, bad
    assert call(Cin=1 << 20, Kw=1 << 20, L=1 << 21) == UNSUPPORTED
    # matrix-core shape without its workspace
    assert call(B=2, Cin=64, L=1024, Cout=32, Kw=3, pad=1) == WORKSPACE
    assert call(B=2, Cin=64, L=1024, Cout=32, Kw=3, pad=1, ws=0x10000, ws_bytes=100) == WORKSPACE
    assert call(B=2, Cin=64, L=1024, Cout=32, Kw=3, pad=1, ws=0x10010, ws_bytes=1 << 30) == WORKSPACE     # misaligned


def test_probes_reject_bad_arguments_on_the_host(lib):
    assert lib.pgk_probe_mfma(0, 1, 10, None, None, None) == INVALID
    assert lib.pgk_probe_mfma(5, 1, 10, 0x1000, None, None) == INVALID
    assert lib.pgk_probe_mfma(0, 1, 0, 0x1000, None, None) == INVALID
    assert lib.pgk_probe_stream_read(None, 1024, 0x1000, None) == INVALID
    assert lib.pgk_probe_stream_read(0x2000, 1000, 0x1000, None) == INVALID     # not a multiple of 16
    assert lib.pgk_probe_stream_read(0x2004, 1024, 0x1000, None) == INVALID     # misaligned

    # the fed matrix-instruction probe: even iteration count, whole 64 KiB pieces
    def fed(copies=1, iters=10, src=0x10000, nbytes=1 << 20, resident=1 << 16, every=0, clock=0x4000):
        return lib.pgk_probe_mfma_fed(copies, iters, src, nbytes, resident, every, clock, None, None)
    assert fed(clock=None) == INVALID and fed(clock=0x4004) == INVALID
    assert fed(iters=0) == INVALID and fed(iters=3) == INVALID and fed(iters=(1 << 20) + 2) == INVALID
    assert fed(src=None) == INVALID and fed(src=0x10008) == INVALID
    assert fed(nbytes=1000) == INVALID and fed(nbytes=(1 << 16) + 16) == INVALID
    assert fed(resident=0) == INVALID and fed(resident=1 << 21) == INVALID and fed(resident=100) == INVALID
    assert fed(every=-1) == INVALID

    # the phase probe: both large-tile instances, 16 words of stamps per output tile
    F32, BF16 = gen.F32, gen.BF16
    wgs = ctypes.c_int32(-1)

    def phases(A=0x1000, B=0x2000, C=0x3000, M=512, N=512, K=256, act=0, dtype=BF16, stamps=0x4000, nbytes=1 << 20):
        return lib.pgk_probe_gemm_phases(A, B, None, C, None, M, N, K, act, dtype, stamps, nbytes, ctypes.byref(wgs), None)
    assert phases(A=None) == INVALID and phases(stamps=None) == INVALID and phases(stamps=0x4004) == INVALID
    assert phases(dtype=7) == INVALID and phases(act=9) == INVALID
    assert phases(A=0x1008) == UNSUPPORTED                       # operands must sit on 16-byte boundaries
    assert phases(N=511) == UNSUPPORTED                          # bf16 rows on 4-byte boundaries
    assert phases(nbytes=4 * 16 * 8 - 1) == WORKSPACE and wgs.value == 4       # 2 x 2 tiles of 256 x 256
    assert phases(dtype=F32, nbytes=16 * 16 * 8 - 1) == WORKSPACE and wgs.value == 16   # 4 x 4 tiles of 128 x 128


def test_python_binding_validates_before_calling(lib):
    import torch
    a = torch.zeros(2, 3)
    with pytest.raises(ValueError):
        binding.gemm_fused(a, torch.zeros(3, 2), None, 0)      # host tensors are refused
    with pytest.raises(ValueError):
        binding._shape(torch.zeros(2, 3), torch.zeros(4, 2))
    with pytest.raises(ValueError):
        binding.reduce_max(torch.zeros(2, 3), 0)


def test_python_binding_validates_outputs_and_workspace(lib):
    """Caller-supplied outputs and workspaces are checked before their pointers reach the C ABI:
    device, dtype, contiguity, element count.  (Host tensors stand in here: the device check is
    the first to fire, the others are exercised on the checker itself.)"""
    import torch
    dev = torch.device("cpu")
    ok = torch.zeros(2, 3, 4)

    class Fake:      # what _check_out looks at, with a switchable is_cuda
        def __init__(self, t, is_cuda=True, device=dev):
            self.t, self.is_cuda, self.device = t, is_cuda, device
            self.dtype, self.shape = t.dtype, t.shape
        def is_contiguous(self): return self.t.is_contiguous()
        def numel(self): return self.t.numel()
        def dim(self): return self.t.dim()
        def data_ptr(self): return self.t.data_ptr()

    chk = binding._check_out
    orig = torch.Tensor
    try:
        binding.torch.Tensor = Fake            # isinstance check of the helper
        assert chk(Fake(ok), "out", (2, 3, 4), torch.float32, dev).t is ok
        assert chk(Fake(ok.view(6, 4)), "out", (2, 3, 4), torch.float32, dev) is not None     # same elements, flattened
        with pytest.raises(ValueError):
            chk(Fake(ok, is_cuda=False), "out", (2, 3, 4), torch.float32, dev)
        with pytest.raises(ValueError):
            chk(Fake(ok, device=torch.device("meta")), "out", (2, 3, 4), torch.float32, dev)
        with pytest.raises(TypeError):
            chk(Fake(ok.double()), "out", (2, 3, 4), torch.float32, dev)
        with pytest.raises(ValueError):
            chk(Fake(ok.transpose(1, 2)), "out", (2, 4, 3), torch.float32, dev)            # strided view
        with pytest.raises(ValueError):
            chk(Fake(ok[:, :2]), "out", (2, 2, 4), torch.float32, dev)                       # not contiguous
        with pytest.raises(ValueError):
            chk(Fake(torch.zeros(2, 3, 3)), "out", (2, 3, 4), torch.float32, dev)            # too small
        with pytest.raises(ValueError):
            chk(Fake(torch.zeros(4, 3, 4)), "out", (2, 3, 4), torch.float32, dev)            # too large is refused too
        wchk = binding._check_workspace
        assert wchk(None, 0, dev) == (None, 0)
        with pytest.raises(ValueError):
            wchk(None, 16, dev)
        with pytest.raises(ValueError):
            wchk(Fake(torch.zeros(64)), 16, dev)                                              # not uint8
        with pytest.raises(ValueError):
            wchk(Fake(torch.zeros(64, dtype=torch.uint8), is_cuda=False), 16, dev)
        ptr, n = wchk(Fake(torch.zeros(64, dtype=torch.uint8)), 16, dev)
        assert n == 64
    finally:
        binding.torch.Tensor = orig


def test_plan_is_consistent_on_random_shapes(lib):
    """pgk_gemm_plan on seeded random shapes of every size class: the tile is one of the table's,
    the workgroup count is tiles x batch x slices, slices stay within their limits and keep at
    least 16 K tiles each, and only small problems are left to the bounds-checked kernel."""
    rng = np.random.default_rng(7)
    tiles = {gen.BF16: {(256, 256, 64), (128, 128, 64), (256, 128, 64), (128, 256, 64), (128, 32, 64), (32, 128, 64)},
             gen.F32: {(128, 128, 32), (64, 64, 32), (128, 32, 32), (32, 128, 32), (32, 32, 32)}}
    for n in range(3000):
        dtype = gen.BF16 if rng.integers(2) else gen.F32
        hi = [40, 300, 3000, 40000][n % 4]
        M, N, K = (int(rng.integers(1, hi)) for _ in range(3))
        if n % 7 == 0:
            K = int(rng.integers(1, 400000))
        batch = int(rng.integers(1, 5)) if n % 3 == 0 else 1
        bt = bool(rng.integers(2))
        p = binding.gemm_plan(M, N, K, batch, dtype, b_transposed=bt)
        what = (dtype, M, N, K, batch, bt, p)
        bm, bn, bk = p["tile"]
        assert p["workgroups"] == -(-M // bm) * -(-N // bn) * batch * p["slices"], what
        assert 1 <= p["slices"] <= 32, what
        if p["matrix_core"]:
            assert p["tile"] in tiles[dtype], what
            if p["slices"] > 1:
                assert -(-K // bk) // p["slices"] >= 16, what
            if (bm, bn) == (32, 32):
                assert dtype == gen.F32 and not bt and M > 32 and N > 32 and K % 4 == 0 and N % 4 == 0 and 64 <= K < 1024, what
                assert -(-M // 64) * -(-N // 64) * batch <= 64 and p["slices"] == 1, what
            elif bm == 32:
                assert M <= 32, what
            elif bn == 32:
                assert N <= 32 and M > 32, what
        else:
            assert p["tile"] == (64, 64, 16) and p["slices"] == 1, what
            assert M * N * K < 262144 or (M < 16 and N < 16 and K < 1024), what
