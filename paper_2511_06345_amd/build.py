"""Builds libpgk.so (HIP, gfx950 only) next to this file."""
from __future__ import annotations

import json
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpgk.so")
OBJ_DIR = os.path.join(HERE, "_build")
# what the compiler reports per kernel (registers, scratch, LDS, waves per SIMD), written at
# build time next to the library; the profile harness reads it
RESOURCES = os.path.join(HERE, "kernel_resources.json")
# hash of the sources the library was built from (tests compare it with the sources as they stand)
BUILT_FROM = os.path.join(HERE, "libpgk.built_from")


def source_hash() -> str:
    """A short hash of csrc/*.hip and *.h as they stand."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.h"))):
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]

SOURCES = ["pgk_api.hip", "pgk_gemm_mfma.hip", "pgk_gemm_mfma_conv.hip", "pgk_gemm_tiny.hip", "pgk_gemm_guarded.hip", "pgk_reduce.hip", "pgk_reduce_max.hip",
           "pgk_probe.hip", "pgk_conv.hip", "pgk_pack.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # one remark block per kernel with its register, scratch and LDS use
    "-Rpass-analysis=kernel-resource-usage",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


_REMARK = re.compile(r"remark:\s+(Function Name|TotalSGPRs|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|"
                     r"Occupancy \[waves/SIMD\]|SGPRs Spill|VGPRs Spill|LDS Size \[bytes/block\]):\s+(\S+)")
_REMARK_KEY = {"TotalSGPRs": "sgprs", "VGPRs": "vgprs", "AGPRs": "agprs", "ScratchSize [bytes/lane]": "scratch_bytes_per_lane",
               "Occupancy [waves/SIMD]": "waves_per_simd", "SGPRs Spill": "sgpr_spills", "VGPRs Spill": "vgpr_spills",
               "LDS Size [bytes/block]": "lds_bytes_per_workgroup"}


def parse_resource_remarks(text: str) -> dict:
    """{mangled kernel name: {vgprs, agprs, sgprs, ...}} from -Rpass-analysis=kernel-resource-usage output."""
    out, cur = {}, None
    for key, val in _REMARK.findall(text):
        if key == "Function Name":
            cur = out.setdefault(val, {})
        elif cur is not None:
            cur[_REMARK_KEY[key]] = int(val)
    return out


def _demangle(names):
    for tool in ("/opt/rocm/llvm/bin/llvm-cxxfilt", "llvm-cxxfilt", "c++filt"):
        try:
            res = subprocess.run([tool], input="\n".join(names), capture_output=True, text=True)
        except OSError:
            continue
        if res.returncode == 0:
            return res.stdout.splitlines()
    return list(names)


def _compile(src: str):
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, "-I", CSRC, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0 or "error:" in res.stderr:
        raise RuntimeError(f"hipcc failed for {src}:\n{res.stderr}")
    return obj, parse_resource_remarks(res.stderr)


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link libpgk.so.  Always recompiles."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    built_from = source_hash()
    if os.path.exists(BUILT_FROM):
        os.remove(BUILT_FROM)
    with ThreadPoolExecutor(max_workers=6) as ex:
        compiled = list(ex.map(_compile, SOURCES))
    objs = [c[0] for c in compiled]
    resources = {}
    for _, r in compiled:
        resources.update(r)
    mangled = sorted(resources)
    table = {plain: dict(resources[m], mangled=m) for m, plain in zip(mangled, _demangle(mangled))}
    with open(RESOURCES, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    # every symbol must resolve: load the library with immediate binding -- in a child process,
    # so that this process does not end up with the system's HIP runtime loaded ahead of the one
    # torch brings along (two runtimes in one process: launches then fail)
    check = "import ctypes, os, sys; ctypes.CDLL(sys.argv[1], mode=getattr(os, 'RTLD_NOW', 2))"
    res = subprocess.run([sys.executable, "-c", check, LIB], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"{LIB} does not load:\n{res.stderr}")
    with open(BUILT_FROM, "w") as f:
        f.write(built_from + "\n")
    if verbose:
        print(f"built {LIB} from sources {built_from}")
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
