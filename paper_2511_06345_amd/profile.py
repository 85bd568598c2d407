"""Profile harness: the metric set a performance engineer looks at, per kernel, as one JSON.

PRAGMA's profiler agent (Section 3.2) hands its optimiser, for every candidate kernel, the
execution time, occupancy, register usage, shared-memory utilisation, matrix-unit activity
and memory throughput, plus any further counters the optimiser asks for by name; the loop
keeps the best code so far together with its profile (Section 3.3) so that every new
attempt is judged against it.  This module is the part of that which is not a language
model: it runs one workload of ``bench.py`` under ``rocprofv3`` -- one run for the kernel
trace, one run per group of hardware counters, each within what the hardware can collect at
once -- and merges the results with what the compiler reported at build time.

    python -m paper_2511_06345_amd.profile --workload c3 [--extra SQ_INSTS_LDS ...]
                                           [--record best.json] [--out DIR]

The harness process itself never touches the GPU: every measurement is a child process.
Nothing here is on the product path.
"""
from __future__ import annotations

import argparse
import csv
import datetime
import glob
import json
import os
import re
import subprocess
import sys
from collections import defaultdict
from typing import Dict, Iterable, List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
BENCH = os.path.join(ROOT, "bench.py")
RESOURCES = os.path.join(HERE, "kernel_resources.json")

# What one rocprofv3 counter run can hold, per hardware block (rocprofv3 does not split a
# request over several passes; asking for more fails).
BLOCK_LIMIT = {"SQ": 8, "TCC": 4, "TCP": 4, "TA": 2, "TD": 2, "GRBM": 2}

# The default metric set.  Each group is one rocprofv3 run and stays within BLOCK_LIMIT:
# the derived metrics of "sq" use five SQ counters and GRBM_GUI_ACTIVE, FETCH_SIZE three TCC
# counters, WRITE_SIZE two, the hit / miss pair two.
DEFAULT_GROUPS = [
    ("sq", ["MfmaUtil", "OccupancyPercent", "LdsUtil", "LDSBankConflict", "VALUBusy"]),
    ("fetch", ["FETCH_SIZE"]),
    ("write", ["WRITE_SIZE"]),
    ("l2", ["TCC_HIT_sum", "TCC_MISS_sum"]),
]

MI355X = {"cus": 256, "simds_per_cu": 4, "max_waves_per_simd": 8, "lds_bytes_per_cu": 160 * 1024,
          "hbm_peak_gbs": 8000.0, "mfma_peak_tflops": {"bf16": 2500.0, "f32": 157.3}}


# ----------------------------------------------------------------------------- planning

def counter_block(name: str) -> Optional[str]:
    """Hardware block of a raw counter name (SQ_..., TCC_..., ...), None for a derived metric."""
    m = re.match(r"^(SQ|TCC|TCP|TA|TD|GRBM)_", name)
    return m.group(1) if m else None


def _base(name: str) -> str:
    return re.sub(r"_(sum|avr|min|max)$", "", name)


def plan_extra_passes(extra: Sequence[str]) -> List[List[str]]:
    """Packs user-named counters into runs.  Raw counters of a block share a run up to that
    block's limit (the _sum/_avr/_min/_max forms of one counter count once); a derived metric
    gets a run of its own, since the raw counters behind it are not known here."""
    passes: List[List[str]] = []
    used: List[Dict[str, set]] = []
    for name in dict.fromkeys(extra):
        blk = counter_block(name)
        if blk is None:
            passes.append([name])
            used.append({"*": {name}})
            continue
        for p, u in zip(passes, used):
            if "*" in u:
                continue
            have = u.setdefault(blk, set())
            if _base(name) in have or len(have) < BLOCK_LIMIT[blk]:
                have.add(_base(name))
                p.append(name)
                break
        else:
            passes.append([name])
            used.append({blk: {_base(name)}})
    return passes


# ----------------------------------------------------------------------------- running

def _rocprof(mode: Sequence[str], out_dir: str, tag: str, program: Sequence[str], limit_s: int, log_path: str) -> None:
    """One rocprofv3 run as a child process, from /tmp, the program itself after `--`."""
    cmd = ["timeout", "-s", "KILL", str(limit_s), "rocprofv3", *mode, "--output-format", "csv",
           "-d", out_dir, "-o", tag, "--", *program]
    env = dict(os.environ, TMPDIR="/tmp")
    os.makedirs(out_dir, exist_ok=True)
    with open(log_path, "w") as log:
        res = subprocess.run(cmd, cwd="/tmp", env=env, stdout=log, stderr=subprocess.STDOUT)
    if res.returncode != 0:
        tail = "".join(open(log_path).readlines()[-15:])
        raise RuntimeError(f"rocprofv3 run '{tag}' failed with status {res.returncode}:\n{tail}")


def trace_run(out_dir: str, program: Sequence[str], limit_s: int) -> None:
    _rocprof(["--kernel-trace", "--stats"], out_dir, "trace", program, limit_s, os.path.join(out_dir, "trace.log"))


def counter_run(out_dir: str, tag: str, counters: Sequence[str], program: Sequence[str], limit_s: int) -> None:
    _rocprof(["--pmc", *counters], out_dir, tag, program, limit_s, os.path.join(out_dir, tag + ".log"))


# ----------------------------------------------------------------------------- parsing

def _find(out_dir: str, suffix: str) -> Optional[str]:
    hits = sorted(glob.glob(os.path.join(out_dir, "**", "*" + suffix), recursive=True))
    return hits[0] if hits else None


def is_library_kernel(name: str) -> bool:
    return "pgk::" in name


def parse_kernel_trace(path: str, warmup_calls: int = 0) -> Dict[str, dict]:
    """Per kernel: calls, average / min / max duration in ns over the dispatches after the
    first `warmup_calls` of that kernel, and the launch resources the trace carries."""
    per: Dict[str, list] = defaultdict(list)
    static: Dict[str, dict] = {}
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            name = row["Kernel_Name"]
            per[name].append(int(row["End_Timestamp"]) - int(row["Start_Timestamp"]))
            if name not in static:
                static[name] = {
                    "workgroup_size": int(row["Workgroup_Size_X"]) * int(row["Workgroup_Size_Y"]) * int(row["Workgroup_Size_Z"]),
                    "grid_size": int(row["Grid_Size_X"]) * int(row["Grid_Size_Y"]) * int(row["Grid_Size_Z"]),
                    "lds_bytes_per_workgroup": int(row["LDS_Block_Size"]),
                    "scratch_bytes_per_lane": int(row["Scratch_Size"]),
                    "trace_vgprs": int(row["VGPR_Count"]), "trace_agprs": int(row["Accum_VGPR_Count"]),
                    "trace_sgprs": int(row["SGPR_Count"]),
                }
    out = {}
    for name, d in per.items():
        d = d[warmup_calls:] if len(d) > warmup_calls else d
        out[name] = dict(static[name], calls=len(d), avg_ns=sum(d) / len(d), min_ns=min(d), max_ns=max(d))
    return out


def parse_counters(path: str) -> Dict[str, Dict[str, float]]:
    """{kernel: {counter: mean over dispatches}} from a counter_collection.csv."""
    acc: Dict[str, Dict[str, list]] = defaultdict(lambda: defaultdict(list))
    with open(path, newline="") as f:
        for row in csv.DictReader(f):
            acc[row["Kernel_Name"]][row["Counter_Name"]].append(float(row["Counter_Value"]))
    return {k: {c: sum(v) / len(v) for c, v in d.items()} for k, d in acc.items()}


def load_resources(path: str = RESOURCES) -> Dict[str, dict]:
    if not os.path.exists(path):
        return {}
    with open(path) as f:
        return json.load(f)


def _squash(name: str) -> str:
    return re.sub(r"\s+", "", name)


def match_resources(kernel: str, table: Dict[str, dict]) -> Optional[dict]:
    """The compiler's record of a traced kernel (names compared without white space)."""
    key = _squash(kernel)
    for name, rec in table.items():
        if _squash(name) == key:
            return rec
    return None


# ----------------------------------------------------------------------------- merging

def occupancy_limits(vgprs_total: int, lds_bytes: int, workgroup_size: int) -> dict:
    """Waves per SIMD that fit, by registers and by LDS (gfx950: 512 registers per lane and
    SIMD in blocks of 8, 160 KiB of LDS per CU, at most 8 waves per SIMD)."""
    hw = MI355X
    alloc = max(8, -(-vgprs_total // 8) * 8)
    by_regs = min(hw["max_waves_per_simd"], 512 // alloc)
    waves_per_wg = max(1, -(-workgroup_size // 64))
    if lds_bytes > 0:
        wgs = hw["lds_bytes_per_cu"] // lds_bytes
        by_lds = min(hw["max_waves_per_simd"], (wgs * waves_per_wg) // hw["simds_per_cu"])
    else:
        by_lds = hw["max_waves_per_simd"]
    return {"by_registers": by_regs, "by_lds": by_lds, "waves_per_simd": min(by_regs, by_lds),
            "max_waves_per_simd": hw["max_waves_per_simd"]}


def merge(trace: Dict[str, dict], counters: Dict[str, Dict[str, float]], resources: Dict[str, dict],
          fetch_scale: float, write_scale: float, all_kernels: bool = False) -> List[dict]:
    """One record per kernel with the default metric set filled in from what was measured."""
    out = []
    for name, t in trace.items():
        if not all_kernels and not is_library_kernel(name):
            continue
        rec = {"kernel": name, "calls": t["calls"], "time_us": t["avg_ns"] / 1e3, "time_us_min": t["min_ns"] / 1e3,
               "time_us_max": t["max_ns"] / 1e3, "workgroup_size": t["workgroup_size"],
               "workgroups": t["grid_size"] // max(1, t["workgroup_size"])}
        res = match_resources(name, resources)
        if res:
            regs = {"vgprs": res["vgprs"], "agprs": res["agprs"], "sgprs": res["sgprs"],
                    "scratch_bytes_per_lane": res["scratch_bytes_per_lane"],
                    "vgpr_spills": res["vgpr_spills"], "sgpr_spills": res["sgpr_spills"], "source": "compiler"}
            lds = res["lds_bytes_per_workgroup"]
            total = res["vgprs"] + res["agprs"]
        else:
            regs = {"vgprs": t["trace_vgprs"], "agprs": t["trace_agprs"], "sgprs": t["trace_sgprs"],
                    "scratch_bytes_per_lane": t["scratch_bytes_per_lane"], "source": "kernel trace"}
            lds = t["lds_bytes_per_workgroup"]
            total = t["trace_vgprs"] + t["trace_agprs"]
        rec["registers"] = regs
        rec["lds"] = {"bytes_per_workgroup": lds, "fraction_of_cu": lds / MI355X["lds_bytes_per_cu"]}
        rec["occupancy"] = occupancy_limits(total, lds, t["workgroup_size"])
        c = counters.get(name, {})
        if "OccupancyPercent" in c:
            rec["occupancy"]["measured_percent"] = c["OccupancyPercent"]
        if "MfmaUtil" in c:
            rec["matrix_unit_busy_percent"] = c["MfmaUtil"]
        if "LdsUtil" in c:
            rec["lds"]["busy_percent"] = c["LdsUtil"]
        if "LDSBankConflict" in c:
            rec["lds"]["bank_conflict_percent"] = c["LDSBankConflict"]
        if "VALUBusy" in c:
            rec["vector_alu_busy_percent"] = c["VALUBusy"]
        mem = {}
        if "FETCH_SIZE" in c:
            mem["read_bytes"] = c["FETCH_SIZE"] * 1024.0 * fetch_scale
        if "WRITE_SIZE" in c:
            mem["written_bytes"] = c["WRITE_SIZE"] * 1024.0 * write_scale
        if "read_bytes" in mem and "written_bytes" in mem:
            mem["gb_per_s"] = (mem["read_bytes"] + mem["written_bytes"]) / t["avg_ns"]
            mem["fraction_of_hbm_peak"] = mem["gb_per_s"] / MI355X["hbm_peak_gbs"]
        if "TCC_HIT_sum" in c and "TCC_MISS_sum" in c and c["TCC_HIT_sum"] + c["TCC_MISS_sum"] > 0:
            mem["l2_hit_percent"] = 100.0 * c["TCC_HIT_sum"] / (c["TCC_HIT_sum"] + c["TCC_MISS_sum"])
        if mem:
            rec["memory"] = mem
        known = {"OccupancyPercent", "MfmaUtil", "LdsUtil", "LDSBankConflict", "VALUBusy", "FETCH_SIZE",
                 "WRITE_SIZE", "TCC_HIT_sum", "TCC_MISS_sum"}
        extra = {k: v for k, v in c.items() if k not in known}
        if extra:
            rec["extra_counters"] = extra
        out.append(rec)
    out.sort(key=lambda r: -r["time_us"] * r["calls"])
    return out


def copy_scale(counters: Dict[str, Dict[str, float]], counter: str, bytes_per_copy: float) -> Optional[float]:
    """Scale factor of FETCH_SIZE / WRITE_SIZE from a plain device-to-device copy of known size."""
    for name, c in counters.items():
        if "copyBuffer" in name and counter in c and c[counter] > 0:
            return bytes_per_copy / (c[counter] * 1024.0)
    return None


# ----------------------------------------------------------------------------- best so far

def update_record(path: str, workload: str, profile: dict) -> dict:
    """Keeps, per workload, the fastest profile seen (by time of one step); returns how this
    run compares with it."""
    table = {}
    if os.path.exists(path):
        with open(path) as f:
            table = json.load(f)
    best = table.get(workload)
    now = profile["step_time_us"]
    verdict = {"previous_best_us": best["step_time_us"] if best else None}
    if best is None or now < best["step_time_us"]:
        table[workload] = profile
        verdict["is_new_best"] = True
        verdict["change_percent"] = None if best is None else 100.0 * (now - best["step_time_us"]) / best["step_time_us"]
        os.makedirs(os.path.dirname(os.path.abspath(path)), exist_ok=True)
        with open(path, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
    else:
        verdict["is_new_best"] = False
        verdict["change_percent"] = 100.0 * (now - best["step_time_us"]) / best["step_time_us"]
        verdict["best_kernels"] = best["kernels"]
    return verdict


# ----------------------------------------------------------------------------- driver

def profile_workload(workload: str, out_dir: str, extra: Sequence[str] = (), steps: int = 20, warmup: int = 5,
                     calibrate: bool = True, limit_s: int = 240, all_kernels: bool = False) -> dict:
    os.makedirs(out_dir, exist_ok=True)
    program = ["python3", BENCH, "--workload", workload, "--steps", str(steps), "--warmup", str(warmup),
               "--no-cpu-baseline", "--no-ceilings", "--headline-only"]
    t_dir = os.path.join(out_dir, "trace")
    trace_run(t_dir, program, limit_s)
    trace = parse_kernel_trace(_find(t_dir, "kernel_trace.csv"), warmup_calls=warmup)
    bench_line = None
    for line in open(os.path.join(t_dir, "trace.log")):
        if line.startswith("{"):
            bench_line = json.loads(line)

    counters: Dict[str, Dict[str, float]] = defaultdict(dict)
    groups = list(DEFAULT_GROUPS) + [(f"extra{i}", p) for i, p in enumerate(plan_extra_passes(extra))]
    for tag, names in groups:
        c_dir = os.path.join(out_dir, tag)
        counter_run(c_dir, tag, names, program, limit_s)
        for kernel, vals in parse_counters(_find(c_dir, "counter_collection.csv")).items():
            counters[kernel].update(vals)

    fetch_scale, write_scale, how = 2.0, 1.0, "defaults (FETCH_SIZE counts half of a copy's bytes on this chip)"
    if calibrate:
        cal = ["python3", BENCH, "--copy-calibration"]
        one_gib = float(1 << 30)
        scales = {}
        for tag, ctr in (("cal_fetch", "FETCH_SIZE"), ("cal_write", "WRITE_SIZE")):
            c_dir = os.path.join(out_dir, tag)
            counter_run(c_dir, tag, [ctr], cal, limit_s)
            scales[ctr] = copy_scale(parse_counters(_find(c_dir, "counter_collection.csv")), ctr, one_gib)
        if scales["FETCH_SIZE"] and scales["WRITE_SIZE"]:
            fetch_scale, write_scale = scales["FETCH_SIZE"], scales["WRITE_SIZE"]
            how = "measured on a plain 1 GiB device-to-device copy in this run"

    kernels = merge(trace, counters, load_resources(), fetch_scale, write_scale, all_kernels)
    step_us = sum(k["time_us"] * k["calls"] for k in kernels) / max(1, steps)
    return {
        "workload": workload,
        "sources": kernel_source_hash(),
        "when": datetime.datetime.now().isoformat(timespec="seconds"),
        "step_time_us": step_us,
        "kernels": kernels,
        "counter_scale": {"FETCH_SIZE": fetch_scale, "WRITE_SIZE": write_scale, "source": how},
        "bench": {k: bench_line[k] for k in ("metric", "value", "unit", "ms_per_step", "dtype")} if bench_line else None,
        "runs": ["trace"] + [g[0] for g in groups] + (["cal_fetch", "cal_write"] if calibrate else []),
    }


def kernel_source_hash() -> str:
    """A short hash of the kernel sources as they stand (csrc/*.hip, *.h): counter values taken from
    one version of the kernels say nothing about another, so every stored traffic figure carries it."""
    from .build import source_hash
    return source_hash()


_TRAFFIC_RE = re.compile(r"^traffic-record: workload=(\S+) sources=(\S+) bytes=(\d+) kernel=(.+)$")


def traffic_record_line(workload: str, sources: str, nbytes: float, kernel: str) -> str:
    return f"traffic-record: workload={workload} sources={sources} bytes={int(round(nbytes))} kernel={kernel}"


def read_traffic_records(profiles_dir: str) -> List[dict]:
    """Every traffic-record line of the summaries under `profiles_dir` (written by to_markdown)."""
    out = []
    for path in sorted(glob.glob(os.path.join(profiles_dir, "*.md"))):
        with open(path) as f:
            for line in f:
                m = _TRAFFIC_RE.match(line.strip().strip("`"))
                if m:
                    out.append({"workload": m.group(1), "sources": m.group(2), "bytes": int(m.group(3)),
                                "kernel": m.group(4).strip(), "file": os.path.basename(path)})
    return out


def stored_traffic(workload: str, kernel_substring: str, profiles_dir: Optional[str] = None) -> Optional[int]:
    """L2 <-> fabric bytes per launch of the kernel whose name contains `kernel_substring` on `workload`,
    from a summary taken with the kernel sources as they are now; None when there is none (then the
    figure would describe other code)."""
    now = kernel_source_hash()
    for rec in read_traffic_records(profiles_dir or os.path.join(ROOT, "profiles")):
        if rec["workload"] == workload and rec["sources"] == now and _squash(kernel_substring) in _squash(rec["kernel"]):
            return rec["bytes"]
    return None


def to_markdown(prof: dict, command: str) -> str:
    """A short text summary of one profile (what profiles/*_metric_set.md hold)."""
    w = prof["workload"]
    sc = prof["counter_scale"]
    out = [f"# Metric set of workload {w} (per kernel) — profile harness over rocprofv3\n",
           "Command (one MI355X; the harness starts one rocprofv3 run for the kernel trace, one per counter group —",
           ", ".join(f"`{g}` = {' '.join(names)}" for g, names in DEFAULT_GROUPS) + " —",
           f"and two calibration runs on a plain 1 GiB copy):\n",
           f"    {command}\n",
           f"Counter scale factors ({sc['source']}): FETCH_SIZE x {sc['FETCH_SIZE']:.4f}, WRITE_SIZE x {sc['WRITE_SIZE']:.4f}.",
           f"Step time (sum of the library's kernels, profiler attached): {prof['step_time_us']:.1f} us.\n"]
    for k in prof["kernels"]:
        r, l, o, m = k["registers"], k["lds"], k["occupancy"], k.get("memory", {})
        out += [f"## `{k['kernel']}`\n", "| metric | value |", "|---|---|",
                f"| time per launch | {k['time_us']:.1f} us (min {k['time_us_min']:.1f}, max {k['time_us_max']:.1f}; {k['calls']} launches) |",
                f"| launch | {k['workgroups']} workgroups of {k['workgroup_size']} threads |",
                f"| registers ({r['source']}) | {r['vgprs']} VGPR + {r['agprs']} AGPR, {r['sgprs']} SGPR, scratch "
                f"{r['scratch_bytes_per_lane']} B/lane, spills {r.get('vgpr_spills', 0)} VGPR / {r.get('sgpr_spills', 0)} SGPR |",
                f"| LDS | {l['bytes_per_workgroup']} B per workgroup = {100 * l['fraction_of_cu']:.0f} % of a CU; busy "
                f"{l.get('busy_percent', 0):.1f} %, bank-conflict stall {l.get('bank_conflict_percent', 0):.2f} % |",
                f"| occupancy | {o['waves_per_simd']} of {o['max_waves_per_simd']} waves per SIMD fit (registers allow "
                f"{o['by_registers']}, LDS {o['by_lds']}); measured {o.get('measured_percent', 0):.1f} % |",
                f"| matrix unit busy (MfmaUtil) | {k.get('matrix_unit_busy_percent', 0):.1f} % |",
                f"| vector ALU busy | {k.get('vector_alu_busy_percent', 0):.1f} % |"]
        if "gb_per_s" in m:
            out.append(f"| memory traffic (L2 <-> fabric) | read {m['read_bytes'] / 1e6:.1f} MB + written {m['written_bytes'] / 1e6:.1f} MB "
                       f"per launch = {m['gb_per_s']:.0f} GB/s ({100 * m['fraction_of_hbm_peak']:.1f} % of 8 TB/s); L2 hit rate "
                       f"{m.get('l2_hit_percent', 0):.1f} % |")
        for name, v in sorted(k.get("extra_counters", {}).items()):
            out.append(f"| {name} | {v:.6g} |")
        out.append("")
        if "gb_per_s" in m:
            # one line a program can read back (bench.py: roofline.traffic), tied to the kernel sources
            out += ["`" + traffic_record_line(w, prof.get("sources", kernel_source_hash()),
                                              m["read_bytes"] + m["written_bytes"], k["kernel"]) + "`", ""]
    return "\n".join(out)


def main(argv: Optional[Iterable[str]] = None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--workload", default="c3")
    ap.add_argument("--extra", nargs="*", default=[], help="further rocprofv3 counter names")
    ap.add_argument("--out", default=os.path.join(ROOT, "gpurun_out", "profile"))
    ap.add_argument("--record", default=None, help="JSON file keeping the best profile so far per workload")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-calibration", action="store_true")
    ap.add_argument("--all-kernels", action="store_true", help="also report kernels that are not the library's")
    ap.add_argument("--markdown", default=None, help="also write a short text summary of the profile to this file")
    args = ap.parse_args(list(argv) if argv is not None else None)
    prof = profile_workload(args.workload, os.path.join(args.out, args.workload), args.extra, args.steps, args.warmup,
                            not args.no_calibration, all_kernels=args.all_kernels)
    if args.record:
        prof["against_best"] = update_record(args.record, args.workload, {k: prof[k] for k in ("workload", "when", "step_time_us", "kernels")})
    if args.markdown:
        cmd = f"python3 bench.py --profile --workload {args.workload}" + (" --extra-counters " + " ".join(args.extra) if args.extra else "")
        os.makedirs(os.path.dirname(os.path.abspath(args.markdown)), exist_ok=True)
        with open(args.markdown, "w") as f:
            f.write(to_markdown(prof, cmd))
    print(json.dumps(prof), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
