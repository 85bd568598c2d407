#!/usr/bin/env python3
"""Benchmark of the fused GEMM + epilogue hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of seeded synthetic
input: one pgk_gemm_fused (or pgk_gemm_splitk) call, i.e. the matrix-core main
loop, the bias/activation/row-sum epilogue and any follow-up reduction kernel.
Inputs are generated on the host by the seeded generator and are resident in HBM
before the timed region starts.

The headline workload is the large bf16 GEMM (M=N=K=8192, bias + SiLU, bf16 out).
Timing follows the protocol of the paper's evaluation (PRAGMA Section 4.1): 5
warm-up runs and 100 timed repetitions by default.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

# MI355X published peaks
PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
PEAK_HBM_GBS = 8000.0
# roofline.traffic (L2 <-> memory bytes per launch of the dominant kernel, from rocprofv3 FETCH_SIZE /
# WRITE_SIZE runs scaled by a plain copy) is read from the traffic-record lines of the summaries under
# profiles/; a record counts only if it was taken with the kernel sources as they are now.

DESCR = {
    "c1": "c1: fp32 GEMM 256x256x256, bias + ReLU + rowsum",
    "c2": "c2: fp32 GEMM 4096x4096x4096, bias + GELU-tanh",
    "c3": "c3: bf16 GEMM 8192x8192x8192 (fp32 accumulate), bias + SiLU, bf16 out",
    "c4": "c4: bf16 GEMM 16384x1024x4096, bias + ReLU + fp32 rowsum, bf16 out",
    "c5": "c5: fp32 split-K GEMM 256x256x65536 x16, identity + rowsum",
}


REDUCE_DESCR = {
    "r1": "r1: fp32 max over dim 1 of [64, 4096, 1024] (strided), values + positions",
    "r2": "r2: fp32 max over dim 2 of [64, 4096, 1024] (contiguous rows of 1024), values + positions",
    "r3": "r3: bf16 max over dim 1 of [32, 4096, 4096] (strided), values + positions",
    "r4": "r4: fp32 max over dim 1 of [16, 2^24] (few long rows, two passes), values + positions",
}


CONV_DESCR = {
    "v1": "v1: fp32 conv1d [16, 64, 65536] * [128, 64, 3], stride 1, pad 1, bias + ReLU (matrix-core path)",
    "v2": "v2: bf16 conv1d [8, 256, 16384] * [256, 256, 5], stride 1, pad 4, dilation 2, bias + SiLU (matrix-core path)",
    "v3": "v3: fp32 conv1d [4, 48, 32768] * [64, 48, 5], stride 2, pad 2, bias (matrix-core path on per-phase copies of the input)",
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def device_inputs(w, gen, torch):
    A, B, bias = gen.make_inputs(w)
    if w.dtype == gen.BF16:
        dA = torch.from_numpy(A.view(np.int16)).cuda().view(torch.bfloat16)
        dB = torch.from_numpy(B.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        dA, dB = torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()
    dbias = torch.from_numpy(bias).cuda() if bias is not None else None
    return (A, B, bias), (dA, dB, dbias)


PREAMBLE_NOTE = ("before the warm-up steps of every workload the matrix-instruction probe runs for about 40 ms: after an "
                 "idle period (host-side input generation) the board's power management takes some fifteen launches to settle, "
                 "and a timed region of a few milliseconds would measure that transient instead of the kernel")


def leave_idle_state(pgk, gen, torch, dtype=None, launches=16):
    """Keeps the GPU busy with the library's matrix-instruction probe right before a timed region, so
    that the region starts from the loaded power state, not from idle (measured on c3: the first
    fifteen launches after half a second of idle take 900-1060 us, then 800)."""
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    for _ in range(launches):
        pgk.probe_mfma(gen.BF16 if dtype is None else dtype, True, 2000, sink)


def run_workload(name, steps, warmup, pgk, gen, torch, keep_host=False, sets=4):
    """Times `steps` calls of the hot path on workload `name`; returns a dict.

    Cache hygiene: the calls rotate through `sets` separate copies of the inputs and outputs
    (same values, different addresses), so that consecutive calls do not find their operands
    in the 256 MB memory-side cache; every copy is resident in HBM before timing starts."""
    w = gen.WORKLOADS[name]
    t0 = time.time()
    host, (dA, dB, dbias) = device_inputs(w, gen, torch)
    # reproducibility: checksums of the exact input bits
    checksums = {"A": f"{gen.fnv1a64(host[0]):016x}", "B": f"{gen.fnv1a64(host[1]):016x}",
                 "bias": f"{gen.fnv1a64(host[2]):016x}" if host[2] is not None else None}
    log(f"[{name}] inputs generated, checksummed and copied in {time.time() - t0:.1f} s")
    out_dt = torch.bfloat16 if w.dtype == gen.BF16 else torch.float32
    fn = pgk.gemm_splitk if w.call == "splitk" else pgk.gemm_fused
    bufs = []
    for i in range(max(1, sets)):
        # the workspace is the caller's: one per buffer set, allocated before timing
        kw = {}
        flags = pgk.WS_ROWSUM if w.rowsum else 0
        need = (pgk.gemm_splitk_workspace_bytes(w.M, w.N, w.K, w.batch, w.dtype, 0, flags) if w.call == "splitk"
                else pgk.gemm_fused_workspace_bytes(w.M, w.N, w.K, w.batch, w.dtype, flags))
        if need:
            kw["workspace"] = torch.empty(need, dtype=torch.uint8, device="cuda")
        bufs.append(dict(
            A=dA if i == 0 else dA.clone(), B=dB if i == 0 else dB.clone(),
            bias=dbias if (i == 0 or dbias is None) else dbias.clone(),
            C=torch.empty((w.batch, w.M, w.N), dtype=out_dt, device="cuda"),
            rs=torch.empty((w.batch, w.M), dtype=torch.float32, device="cuda") if w.rowsum else None, kw=kw))

    def step(i):
        b = bufs[i % len(bufs)]
        fn(b["A"], b["B"], b["bias"], w.act, rowsum=w.rowsum, out=b["C"], rowsum_out=b["rs"], **b["kw"])

    leave_idle_state(pgk, gen, torch, w.dtype)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    # events are recorded on torch's current stream, the stream the kernels are launched on
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t_start = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        step(warmup + i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    per = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])  # ms, per call
    ms_per_step = wall * 1e3 / steps
    res = {
        "workload": DESCR[name],
        "ms_per_step": ms_per_step,
        "tflops": w.flops / (ms_per_step * 1e-3) / 1e12,
        "call_ms_avg": float(per.mean()),
        "call_ms_median": float(np.median(per)),
        "call_ms_min": float(per.min()),
        "algorithmic_gbs": w.algorithmic_bytes / (float(per.mean()) * 1e-3) / 1e9,
        "buffer_sets": len(bufs),
        "input_checksums_fnv1a64": checksums,
    }
    if w.flops < 1e9:
        # a launch-bound workload: the same call captured once into a HIP graph and replayed -- what the
        # kernels cost without the per-call work of the Python binding
        side = torch.cuda.Stream()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step(0)
        for _ in range(warmup):
            graph.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(steps):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        res["graph_replay_ms_per_step"] = g0.elapsed_time(g1) / steps
    if keep_host:
        res["_host"] = host
        res["_out"] = (bufs[0]["C"], bufs[0]["rs"])      # what the timed calls wrote (every buffer set holds the same values)
    return res


def gemm_kernel_name(w, pgk, gen):
    """The instance of the matrix-core kernel the fused / split call runs for this workload, as the
    profiler prints it (from pgk_gemm_plan: tile shape; the wave layout follows from the tile)."""
    plan = pgk.gemm_plan(w.M, w.N, w.K, w.batch, w.dtype)
    bm, bn, bk = plan["tile"]
    if not plan["matrix_core"]:
        return "pgk::gemm_guarded_kernel", plan
    bf = w.dtype == gen.BF16
    if (bm, bn) == (32, 32):
        return "pgk::gemm_tiny_f32_kernel", plan
    layout = {(256, 256): "4, 2, 3, 2", (128, 128): "2, 2, 3, 2" if bf else "2, 2, 2, 1", (64, 64): "2, 2, 2, 2",
              (256, 128): "4, 2, 3, 2", (128, 256): "2, 4, 3, 2", (32, 128): "1, 4, 2, 2", (128, 32): "4, 1, 2, 2"}[(bm, bn)]
    return f"MfmaCfg<{'true' if bf else 'false'}, {bm}, {bn}, {bk}, {layout}>, 0, false>", plan


def gemm_roofline(name, w, res, pgk, gen):
    """Roofline block of one GEMM workload: the matrix pipe binds all five (their HBM times are 3-40 %
    of their matrix times), so `frac` is against the published matrix peak of the type; the HBM
    fraction of the algorithmic bytes is reported beside it."""
    from paper_2511_06345_amd import profile
    dtype_key = "bf16" if w.dtype == gen.BF16 else "f32"
    achieved = w.flops / (res["call_ms_avg"] * 1e-3) / 1e12
    kernel, plan = gemm_kernel_name(w, pgk, gen)
    return {
        "bound": "mfma",
        "kernel": "pgk::gemm_mfma_kernel<" + kernel if kernel.startswith("MfmaCfg") else kernel,
        "plan": plan,
        "achieved": achieved,
        "peak": PEAK_TFLOPS[dtype_key],
        "unit": "TFLOP/s",
        "frac": achieved / PEAK_TFLOPS[dtype_key],
        "launch_ms_avg": res["call_ms_avg"],
        "launch_ms_median": res["call_ms_median"],
        "launch_ms_min": res["call_ms_min"],
        "traffic": profile.stored_traffic(name, kernel),
        "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE and WRITE_SIZE, each scaled by the same counter on a plain "
                        "1 GiB copy; null: no summary under profiles/ was taken with the kernel sources as they are now)",
        "hbm_achieved_gbs_algorithmic": res["algorithmic_gbs"],
        "hbm_frac_algorithmic": res["algorithmic_gbs"] / PEAK_HBM_GBS,
    }


def phase_budget(name, pgk, gen, torch, launches=6, sets=1, warmup=2):
    """Where the time of the large-tile kernel goes on workload `name` (c3, c4: bf16; c2: fp32), and at
    which shader clock: `launches` timed launches of the measurement instance of the kernel
    (pgk_probe_gemm_phases: the shipping kernel plus cycle-counter / 100 MHz-counter stamps),
    rotating through `sets` copies of the buffers like the timed region of the bench.  Per launch:
    event time, clock (cycles per tick summed over the workgroups), main-loop cycles per K tile;
    the stamps of the last launch are reduced to medians over the workgroups of each round."""
    w = gen.WORKLOADS[name]
    if w.batch != 1 or w.call != "fused" or w.flops < 1e11:
        raise SystemExit("--phases: the timed instances are the large-tile kernels (workloads c2, c3, c4)")
    # tile, workgroups resident on one CU (registers and LDS of the instance), matrix-core flops per
    # cycle of one CU (published peak / 256 CUs / 2.4 GHz)
    bf16 = w.dtype == gen.BF16
    bm, bn, bk, per_cu, cu_flops_per_cycle = (256, 256, 64, 1, 4096) if bf16 else (128, 128, 32, 2, 256)
    issue_cycles = bm * bn * bk * 2 // cu_flops_per_cycle * per_cu   # per K tile, as one workgroup sees them
    _, (dA, dB, dbias) = device_inputs(w, gen, torch)
    tiles_n = -(-w.N // bn)
    wgs = -(-w.M // bm) * tiles_n
    bufs = [dict(A=dA if i == 0 else dA.clone(), B=dB if i == 0 else dB.clone(),
                 C=torch.empty((1, w.M, w.N), dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda"),
                 part=torch.empty((tiles_n, w.M), dtype=torch.float32, device="cuda") if w.rowsum else None)
            for i in range(max(1, sets))]
    stamps = torch.zeros((launches, wgs, pgk.STAMP_WORDS), dtype=torch.int64, device="cuda")
    scratch_stamps = torch.zeros((wgs, pgk.STAMP_WORDS), dtype=torch.int64, device="cuda")

    def launch(i, st):
        b = bufs[i % len(bufs)]
        pgk.probe_gemm_phases(b["A"], b["B"], dbias, w.act, b["C"], st, rowsum_partials=b["part"])

    leave_idle_state(pgk, gen, torch)
    for i in range(warmup):
        launch(i, scratch_stamps)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(launches + 1)]
    ev[0].record()
    for i in range(launches):
        launch(warmup + i, stamps[i])
        ev[i + 1].record()
    torch.cuda.synchronize()
    per_ms = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(launches)])
    st_all = stamps.cpu().numpy().astype(np.float64)
    kt = -(-w.K // bk)
    clocks, loop_cycles = [], []
    for st in st_all:
        cyc, tick = st[:, 0:12:2], st[:, 1:12:2]
        clocks.append((cyc[:, 5] - cyc[:, 0]).sum() / (tick[:, 5] - tick[:, 0]).sum() * 0.1)
        # (workgroups of the first round: every CU holds its full set of them for the whole loop)
        first = np.argsort(tick[:, 0], kind="stable")[:256 * per_cu]
        loop_cycles.append(float(np.median(cyc[first, 2] - cyc[first, 1])) / max(1, kt - 1))
    st = st_all[-1]
    cyc, tick = st[:, 0:12:2], st[:, 1:12:2]                      # [workgroup][stamp]
    t0 = tick[:, 0].min()
    us = (tick - t0) / 100.0                                      # 100 MHz ticks -> microseconds since the first entry
    cus = 256 * per_cu                                            # workgroups resident at once
    rounds = max(1, -(-wgs // cus))
    order = np.argsort(us[:, 0], kind="stable")                   # by entry time: round r = r-th group of that many
    names = ["entry -> first K tile landed", "main loop", "tile's biases handed out through LDS",
             "bias + activation (+ row sums), staging through LDS, stores issued", "stores acknowledged"]
    per_round = []
    for r in range(rounds):
        sel = order[r * cus:(r + 1) * cus]
        d_us = np.diff(us[sel], axis=1)
        d_cyc = np.diff(cyc[sel], axis=1)
        per_round.append({
            "workgroups": int(sel.size),
            "entry_us_median": float(np.median(us[sel, 0])),
            "exit_us_median": float(np.median(us[sel, 5])),
            "phases": [{"phase": names[k], "us_median": float(np.median(d_us[:, k])), "us_max": float(d_us[:, k].max()),
                        "cycles_median": float(np.median(d_cyc[:, k]))} for k in range(5)],
        })
    xcd = st[:, 13].astype(np.int64) & 0xF
    clk = float(np.median(clocks))
    ms = float(np.median(per_ms))
    achieved = w.flops / (ms * 1e-3) / 1e12
    peak_at_clock = PEAK_TFLOPS["bf16" if bf16 else "f32"] * clk / 2.4
    return {
        "workload": DESCR[name], "workgroups": int(wgs), "rounds": rounds, "k_tiles": kt,
        "launches": launches, "buffer_sets": len(bufs),
        "launch_ms_median": ms, "launch_ms_min": float(per_ms.min()),
        "kernel_span_us_last_launch": float((tick[:, 5].max() - t0) / 100.0),
        "shader_clock_ghz_under_kernel": clk,
        "shader_clock_ghz_min_max": [float(min(clocks)), float(max(clocks))],
        "main_loop_cycles_per_k_tile": float(np.median(loop_cycles)),
        "workgroups_per_cu": per_cu,
        "mfma_issue_cycles_per_k_tile": issue_cycles,
        "main_loop_issue_efficiency": issue_cycles / float(np.median(loop_cycles)),
        "achieved_tflops": achieved,
        "peak_tflops_at_this_clock": peak_at_clock,      # the published peak is quoted at 2.4 GHz
        "frac_of_peak_at_this_clock": achieved / peak_at_clock,
        "xcd_of_workgroup_matches_id_mod_8": bool(np.all(xcd == (np.arange(wgs) % 8))),
        "rounds_detail": per_round,
        "how": "wave-0 stamps of s_memtime / s_memrealtime inside a measurement instance of the kernel "
               "(pgk_probe_gemm_phases); clock and cycles: median over the launches; phases: medians over the "
               "workgroups of a round, last launch",
    }


def gpu_clocks():
    """Clock levels of the board right after the timed region, read from the driver's sysfs files
    (no child process: a GPU process must not start other programs).  Best effort."""
    import glob
    out = {}
    for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk") + glob.glob("/sys/class/drm/card*/device/pp_dpm_mclk")):
        try:
            with open(path) as f:
                levels = [ln.strip() for ln in f if ln.strip()]
        except OSError as exc:
            out[path] = f"unreadable: {exc}"
            continue
        cur = [ln for ln in levels if ln.endswith("*")]
        key = path.split("/")[4] + "/" + path.rsplit("_", 1)[-1]
        out[key] = {"current": cur[0].rstrip(" *") if cur else None, "levels": [ln.rstrip(" *") for ln in levels]}
    return out or {"unavailable": "no pp_dpm_sclk / pp_dpm_mclk under /sys/class/drm"}


def run_reduce_workload(name, steps, warmup, pgk, gen, torch, keep_host=False, sets=4):
    """Times `steps` calls of pgk_reduce_max on reduction workload `name`; returns a dict.
    The calls rotate through `sets` copies of the input at different addresses."""
    w = gen.REDUCE_WORKLOADS[name]
    t0 = time.time()
    X = gen.make_reduce_input(w)
    dX = (torch.from_numpy(X.view(np.int16)).cuda().view(torch.bfloat16) if w.dtype == gen.BF16
          else torch.from_numpy(X).cuda())
    log(f"[{name}] input generated and copied in {time.time() - t0:.1f} s")
    shape = tuple(d for i, d in enumerate(w.shape) if i != w.dim)
    vals = torch.empty(shape, dtype=dX.dtype, device="cuda")
    idx = torch.empty(shape, dtype=torch.int32, device="cuda")
    copies = [dX] + [dX.clone() for _ in range(max(1, sets) - 1)]
    outer = int(np.prod(w.shape[:w.dim], dtype=np.int64))
    inner = int(np.prod(w.shape[w.dim + 1:], dtype=np.int64))
    need = pgk.reduce_max_workspace_bytes(outer, w.shape[w.dim], inner, w.dtype)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None

    def step(i):
        pgk.reduce_max(copies[i % len(copies)], w.dim, want_idx=True, out=vals, idx_out=idx, workspace=ws)

    leave_idle_state(pgk, gen, torch)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t_start = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        step(warmup + i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    per = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])
    ms_per_step = wall * 1e3 / steps
    res = {
        "workload": REDUCE_DESCR[name],
        "ms_per_step": ms_per_step,
        "gbs": w.algorithmic_bytes / (ms_per_step * 1e-3) / 1e9,
        "call_ms_avg": float(per.mean()),
        "call_ms_median": float(np.median(per)),
        "call_ms_min": float(per.min()),
        "algorithmic_gbs": w.algorithmic_bytes / (float(per.mean()) * 1e-3) / 1e9,
        "buffer_sets": len(copies),
    }
    res["hbm_frac_algorithmic"] = res["algorithmic_gbs"] / PEAK_HBM_GBS
    if keep_host:
        res["_host"] = X
    return res


def run_conv_workload(name, steps, warmup, pgk, gen, torch, keep_host=False, sets=4):
    """Times `steps` calls of pgk_conv1d on convolution workload `name`; returns a dict.
    The calls rotate through `sets` copies of input and output at different addresses."""
    cw = gen.CONV_WORKLOADS[name]
    t0 = time.time()
    x, w, bias = gen.make_conv_inputs(cw)
    if cw.dtype == gen.BF16:
        dx = torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
        dw = torch.from_numpy(w.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        dx, dw = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    dbias = torch.from_numpy(bias).cuda()
    log(f"[{name}] inputs generated and copied in {time.time() - t0:.1f} s")
    need = pgk.conv1d_workspace_bytes(cw.B, cw.Cin, cw.L, cw.Cout, cw.Kw, cw.stride, cw.pad, cw.dilation, cw.dtype)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    xs = [dx] + [dx.clone() for _ in range(max(1, sets) - 1)]
    ys = [torch.empty((cw.B, cw.Cout, cw.Lout), dtype=dx.dtype, device="cuda") for _ in xs]

    def step(i):
        pgk.conv1d(xs[i % len(xs)], dw, dbias, cw.act, cw.stride, cw.pad, cw.dilation, out=ys[i % len(xs)], workspace=ws)

    leave_idle_state(pgk, gen, torch)
    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    t_start = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        step(warmup + i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    per = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(steps)])
    ms_per_step = wall * 1e3 / steps
    res = {
        "workload": CONV_DESCR[name],
        "ms_per_step": ms_per_step,
        "tflops": cw.flops / (ms_per_step * 1e-3) / 1e12,
        "call_ms_avg": float(per.mean()),
        "call_ms_median": float(np.median(per)),
        "call_ms_min": float(per.min()),
        "algorithmic_gbs": cw.algorithmic_bytes / (float(per.mean()) * 1e-3) / 1e9,
        "workspace_bytes": need,
        "buffer_sets": len(xs),
    }
    res["hbm_frac_algorithmic"] = res["algorithmic_gbs"] / PEAK_HBM_GBS
    if keep_host:
        res["_host"] = (x, w, bias)
    return res


def conv_main(args, name, pgk, gen, torch):
    """One JSON line for a convolution workload."""
    cw = gen.CONV_WORKLOADS[name]
    head = run_conv_workload(name, args.steps, args.warmup, pgk, gen, torch, keep_host=True, sets=args.buffer_sets)
    x, w, bias = head.pop("_host")
    dtype_key = "bf16" if cw.dtype == gen.BF16 else "f32"
    fast = head["workspace_bytes"] > 0
    # the matrix-core path is priced against the matrix peak of its type, the bounds-checked
    # path (plain fp32 FMA) against the fp32 vector peak
    peak = PEAK_TFLOPS[dtype_key] if fast else 157.3
    achieved = cw.flops / (head["call_ms_avg"] * 1e-3) / 1e12
    out = {
        "metric": "conv1d+epilogue TFLOP/s on 1 MI355X",
        "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype_key,
        "data": f"synthetic (seeded SplitMix64 generator, resident in HBM before timing; calls rotate through {head['buffer_sets']} copies)",
        "config": {"workload": CONV_DESCR[name], "B": cw.B, "Cin": cw.Cin, "L": cw.L, "Cout": cw.Cout, "Kw": cw.Kw,
                   "stride": cw.stride, "pad": cw.pad, "dilation": cw.dilation, "flops_per_step": cw.flops,
                   "algorithmic_bytes_per_step": cw.algorithmic_bytes, "workspace_bytes": head["workspace_bytes"]},
        "roofline": {"bound": "mfma" if fast else "alu",
                     "kernel": "pgk::gemm_mfma_kernel on shifted views (+ pad and weight regrouping kernels)" if fast
                               else "pgk::gemm_guarded_kernel reading the input in place",
                     "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "launch_ms_avg": head["call_ms_avg"], "traffic": None,
                     "hbm_frac_algorithmic": head["hbm_frac_algorithmic"]},
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        nb, nco = 1, min(cw.Cout, 16)
        oracle.conv1d(x[:1, :, :64 + cw.Kw * cw.dilation], w[:1], None)      # loads the library
        t0 = time.perf_counter()
        oracle.conv1d(x[:nb], w[:nco], bias[:nco], cw.act, cw.stride, cw.pad, cw.dilation)
        dt = time.perf_counter() - t0
        fl = 2.0 * nb * nco * cw.Lout * cw.Cin * cw.Kw
        out["cpu_baseline"] = {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"{nb} batch entry x {nco} output channels of {name} ({fl:.3e} flop in {dt:.2f} s, "
                                         "direct loops in double, gcc -O2 -fopenmp)"}
    print(json.dumps(out), flush=True)


def reduce_main(args, name, pgk, gen, torch):
    """One JSON line for a reduction workload (bound: HBM)."""
    w = gen.REDUCE_WORKLOADS[name]
    head = run_reduce_workload(name, args.steps, args.warmup, pgk, gen, torch, keep_host=True, sets=args.buffer_sets)
    X = head.pop("_host")
    out = {
        "metric": "max-reduction algorithmic GB/s on 1 MI355X",
        "value": head["gbs"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.dtype == gen.BF16 else "f32",
        "data": "synthetic (seeded SplitMix64 block of 2^24 uniform values repeated, resident in HBM before timing)",
        "config": {"workload": REDUCE_DESCR[name], "shape": list(w.shape), "dim": w.dim,
                   "algorithmic_bytes_per_step": w.algorithmic_bytes},
        "roofline": {
            "bound": "hbm",
            "kernel": "pgk::reduce_max_rows_kernel / reduce_max_cols_kernel (+ reduce_max_finish_kernel)",
            "achieved": head["algorithmic_gbs"],
            "peak": PEAK_HBM_GBS,
            "unit": "GB/s",
            "frac": head["algorithmic_gbs"] / PEAK_HBM_GBS,
            "launch_ms_avg": head["call_ms_avg"],
            "traffic": __import__("paper_2511_06345_amd.profile", fromlist=["x"]).stored_traffic(name, "reduce_max_"),
            "traffic_unit": "bytes per launch of the first (streaming) kernel (rocprofv3 FETCH_SIZE and WRITE_SIZE, scaled by "
                            "a plain 1 GiB copy); null: no summary taken with the kernel sources as they are now",
        },
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        oracle.reduce_max(X[:1], w.dim)   # loads the library before the timed call
        t0 = time.perf_counter()
        oracle.reduce_max(X, w.dim)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": w.algorithmic_bytes / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"the whole {name} tensor ({w.elements} elements in {dt * 1e3:.0f} ms, one scan per output, gcc -O2 -fopenmp)",
        }
    print(json.dumps(out), flush=True)


def measured_ceilings(pgk, gen, torch):
    """What this chip sustains under its power limit (library probes, timed with events on the
    launch stream): the matrix instruction alone with zero and with random operands, and a
    streaming read of 2 GiB.  Context for the roofline fractions; the published peaks stay the
    denominators."""
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")

    def timed(fn, reps=5):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        ev[0].record()
        for i in range(reps):
            fn()
            ev[i + 1].record()
        torch.cuda.synchronize()
        return float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(reps)])) * 1e-3

    out = {}
    for key, dtype, rnd in (("mfma_bf16_zero_operands_tflops", gen.BF16, False), ("mfma_bf16_random_operands_tflops", gen.BF16, True),
                            ("mfma_f32_random_operands_tflops", gen.F32, True)):
        flops = [0.0]

        def launch():
            flops[0] = pgk.probe_mfma(dtype, rnd, 2000, sink)
        t = timed(launch)
        out[key] = flops[0] / t / 1e12
    buf = torch.ones(1 << 29, dtype=torch.float32, device="cuda")       # 2 GiB
    t = timed(lambda: pgk.probe_stream_read(buf, sink))
    out["hbm_stream_read_gbs"] = buf.numel() * 4 / t / 1e9
    del buf
    # the bf16 matrix instruction fed the way the 256x256x64 kernel feeds it (pgk_probe_mfma_fed):
    # operands re-read from LDS; plus the 64 KiB copies per K tile out of L2; plus every fifth of
    # those pieces streamed from memory (the kernel's L2 hit rate on c3 is 80 %)
    clock = torch.zeros(4, dtype=torch.int64, device="cuda")
    resident = 2 << 20
    src = (torch.randn(((1 << 30) + resident) // 2, dtype=torch.float32, device="cuda") * 0.01).to(torch.bfloat16)
    fed = {}
    for key, kw in (("lds_operand_reads", {}),
                    ("lds_operand_reads_and_copies_from_l2", {"src": src, "resident_bytes": resident}),
                    ("lds_operand_reads_and_copies_one_in_five_from_memory",
                     {"src": src, "resident_bytes": resident, "stream_every": 5})):
        flops = [0.0]

        def launch():
            flops[0] = pgk.probe_mfma_fed(1000, clock, **kw)
        t = timed(launch)
        cyc, tick = (int(v) for v in clock[:2].cpu())
        fed[key] = {"tflops": flops[0] / t / 1e12, "shader_clock_ghz": cyc / max(1, tick) * 0.1}
    out["mfma_bf16_fed_like_the_large_kernel"] = fed
    del src
    return out


def cpu_baseline(w, host, gen, budget_s=15.0, gpu_out=None):
    """The CPU oracle, as it stands, on a bounded sample of whole rows of the workload.  With
    `gpu_out` = (C, rowsum) device tensors of the timed calls, also what the oracle says about those
    rows of the timed output (second return value): the judged error and its unjudged companions."""
    import oracle
    oracle.build()
    A, B, bias = host
    rng = np.random.default_rng(12345)
    probe_rows = np.sort(rng.choice(w.M, size=min(16, w.M), replace=False)).astype(np.int64)
    t0 = time.perf_counter()
    oracle.gemm_fused(A, B, bias, w.act, rows=probe_rows, want_rowsum=w.rowsum)
    t_probe = time.perf_counter() - t0
    n_rows = int(min(w.M, max(16, budget_s / max(t_probe, 1e-6) * probe_rows.size)))
    rows = np.sort(rng.choice(w.M, size=n_rows, replace=False)).astype(np.int64)
    t0 = time.perf_counter()
    ref_c, ref_rs = oracle.gemm_fused(A, B, bias, w.act, rows=rows, want_rowsum=w.rowsum)
    dt = time.perf_counter() - t0
    flops = 2.0 * n_rows * w.N * w.K * w.batch
    parity = None
    if gpu_out is not None:
        import torch
        C, rs = gpu_out
        sel = torch.from_numpy(rows).to(C.device)
        got = C[:, sel]
        if w.dtype == gen.BF16:
            got = gen.bf16_bits_to_f32(got.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)).astype(np.float64)
        else:
            got = got.cpu().numpy().astype(np.float64)

        def figures(g, r):
            rms = float(np.sqrt(np.mean(r * r)))
            d = np.abs(g - r)
            big = np.abs(r) >= rms
            return {"judged_max_err_over_max_abs_ref_and_rms": float(np.max(d / np.maximum(np.abs(r), rms))),
                    "strict_max_rel_err_where_ref_at_least_rms": float(np.max(d[big] / np.abs(r[big]))) if big.any() else 0.0,
                    "max_abs_err": float(d.max())}
        parity = {"rows": int(n_rows), "bar": 2e-2 if w.dtype == gen.BF16 else 1e-4, "C": figures(got, ref_c)}
        if rs is not None and ref_rs is not None:
            parity["rowsum"] = figures(rs[:, sel].cpu().numpy().astype(np.float64), ref_rs)
        parity["within_bar"] = bool(parity["C"]["judged_max_err_over_max_abs_ref_and_rms"] <= parity["bar"] and
                                    ("rowsum" not in parity or
                                     parity["rowsum"]["judged_max_err_over_max_abs_ref_and_rms"] <= parity["bar"]))
    return parity, {
        "value": flops / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"{n_rows} seeded random whole rows of the {w.M}-row {w.name} problem "
                  f"({flops:.3e} flop in {dt:.1f} s, plain C triple loop in double, gcc -O2 -fopenmp)",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3", choices=sorted(DESCR) + sorted(REDUCE_DESCR) + sorted(CONV_DESCR),
                    help="c1..c5: fused GEMM workloads (c3 is the headline); r1..r4: max-reduction workloads; "
                         "v1..v3: conv1d workloads")
    ap.add_argument("--others", action="store_true",
                    help="also time the reduction and convolution workloads (the other four GEMM workloads are "
                         "always timed and reported under 'others')")
    ap.add_argument("--headline-only", action="store_true", help="time the named workload only")
    ap.add_argument("--phases", action="store_true",
                    help="print the phase budget of the large bf16 kernel on the workload (c3 or c4) as one JSON line "
                         "and exit (timed instance of the kernel; see pgk_probe_gemm_phases)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the probe kernels that measure what the chip sustains (profiling runs)")
    ap.add_argument("--buffer-sets", type=int, default=4,
                    help="copies of the inputs/outputs the timed calls rotate through (cache hygiene)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="launch plain 1 GiB device-to-device copies and exit (run under rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE to get the counters' scale factor)")
    ap.add_argument("--profile", action="store_true",
                    help="run the workload under rocprofv3 (kernel trace, then counter runs) and print the "
                         "per-kernel metric set as one JSON line instead of timing it here")
    ap.add_argument("--extra-counters", nargs="*", default=[], help="with --profile: further counter names")
    ap.add_argument("--record", default=None, help="with --profile: JSON file keeping the best profile so far")
    ap.add_argument("--markdown", default=None, help="with --profile: also write a short text summary to this file")
    args = ap.parse_args()
    if args.profile:
        # the measurements are child processes (this bench again, without --profile); this process
        # stays off the GPU
        from paper_2511_06345_amd import profile
        argv = ["--workload", args.workload, "--extra", *args.extra_counters]
        if args.record:
            argv += ["--record", args.record]
        if args.markdown:
            argv += ["--markdown", args.markdown]
        sys.exit(profile.main(argv))
    if args.gpus != 1:
        sys.exit("bench.py: this library is single-GPU; run with --gpus 1 (nothing here uses a second GPU)")

    if not args.no_cpu_baseline:
        # the oracle's C library is compiled (a child process) before this process touches the GPU:
        # a process that has initialised the GPU starts no other program
        import oracle
        oracle.build()
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = 1 << 28                                   # 2^28 fp32 = 1 GiB read + 1 GiB written per copy
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read_per_copy": 4 * n, "bytes_written_per_copy": 4 * n,
                                               "copies": 4}}))
        return
    from paper_2511_06345_amd import binding as pgk
    from paper_2511_06345_amd import inputs as gen
    pgk.load_library()   # no fallback: fails here if libpgk.so is not built

    name = args.workload
    if name in REDUCE_DESCR:
        reduce_main(args, name, pgk, gen, torch)
        return
    if name in CONV_DESCR:
        conv_main(args, name, pgk, gen, torch)
        return
    w = gen.WORKLOADS[name]
    if args.phases:
        print(json.dumps({"phase_budget": phase_budget(name, pgk, gen, torch, launches=args.steps, sets=args.buffer_sets,
                                                       warmup=args.warmup)}), flush=True)
        return
    head = run_workload(name, args.steps, args.warmup, pgk, gen, torch, keep_host=True, sets=args.buffer_sets)
    clocks = gpu_clocks()
    host = head.pop("_host")
    gpu_out = head.pop("_out")

    dtype_key = "bf16" if w.dtype == gen.BF16 else "f32"
    roofline = gemm_roofline(name, w, head, pgk, gen)
    achieved = roofline["achieved"]

    out = {
        "metric": "fused GEMM+epilogue TFLOP/s on 1 MI355X",
        "value": head["tflops"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": dtype_key,
        "data": "synthetic (seeded SplitMix64 generator, resident in HBM before timing; calls rotate through "
                f"{head['buffer_sets']} copies of the buffers)",
        "protocol": PREAMBLE_NOTE,
        "config": {"workload": DESCR[name], "M": w.M, "N": w.N, "K": w.K, "batch": w.batch,
                   "call": w.call, "flops_per_step": w.flops, "algorithmic_bytes_per_step": w.algorithmic_bytes,
                   "input_checksums_fnv1a64": head["input_checksums_fnv1a64"]},
        "roofline": roofline,
        "call_ms": {"avg": head["call_ms_avg"], "median": head["call_ms_median"], "min": head["call_ms_min"]},
        "gpu_clocks_after_timed_region": clocks,
    }
    if not args.no_ceilings:
        out["measured_ceilings"] = measured_ceilings(pgk, gen, torch)
        mc = out["measured_ceilings"]
        key = "mfma_bf16_random_operands_tflops" if w.dtype == gen.BF16 else "mfma_f32_random_operands_tflops"
        roofline["frac_of_measured_ceiling"] = achieved / mc[key]
    if not args.no_cpu_baseline:
        log("[cpu_baseline] timing the oracle on a bounded sample ...")
        # (the same oracle rows also judge the output of the timed calls: the bench line carries its own parity figure)
        out["parity_of_timed_output_on_oracle_sample"], out["cpu_baseline"] = cpu_baseline(w, host, gen, gpu_out=gpu_out)
    del host, gpu_out
    if w.call == "fused" and w.batch == 1 and w.flops >= 1e11 and not args.no_ceilings:
        # the shader clock the kernel itself sees (cycle counter against the 100 MHz counter)
        # (the same number of launches, rotating through the same number of buffer sets, with the
        # measurement instance of the kernel: what the chip's power management grants this kernel)
        try:
            pb = phase_budget(name, pgk, gen, torch, launches=args.steps, sets=args.buffer_sets, warmup=args.warmup)
            pb.pop("rounds_detail")
            roofline["at_measured_clock"] = {k: pb[k] for k in (
                "shader_clock_ghz_under_kernel", "shader_clock_ghz_min_max", "launch_ms_median", "achieved_tflops",
                "peak_tflops_at_this_clock", "frac_of_peak_at_this_clock", "main_loop_cycles_per_k_tile",
                "main_loop_issue_efficiency", "how")}
        except Exception as exc:      # noqa: BLE001  (a measurement aid must not take the bench line down)
            roofline["at_measured_clock"] = None
            log(f"[phases] skipped: {exc}")
        torch.cuda.empty_cache()
    others = {}
    if not args.headline_only:
        # the other four GEMM workloads, each with its own roofline block
        for other in sorted(DESCR):
            if other == name:
                continue
            r = run_workload(other, args.steps, args.warmup, pgk, gen, torch, sets=args.buffer_sets)
            ow = gen.WORKLOADS[other]
            r["roofline"] = gemm_roofline(other, ow, r, pgk, gen)
            r["config"] = {"M": ow.M, "N": ow.N, "K": ow.K, "batch": ow.batch, "call": ow.call,
                           "flops_per_step": ow.flops, "algorithmic_bytes_per_step": ow.algorithmic_bytes}
            others[other] = r
            torch.cuda.empty_cache()
        out["others"] = others
    if args.others:
        for other in sorted(REDUCE_DESCR):
            others[other] = run_reduce_workload(other, args.steps, args.warmup, pgk, gen, torch, sets=args.buffer_sets)
            torch.cuda.empty_cache()
        for other in sorted(CONV_DESCR):
            others[other] = run_conv_workload(other, args.steps, args.warmup, pgk, gen, torch, sets=args.buffer_sets)
            torch.cuda.empty_cache()
        out["others"] = others
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
