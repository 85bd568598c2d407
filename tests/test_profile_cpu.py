"""Host logic of the profile harness (no GPU, no profiler run): packing counters into runs
within the hardware limits, parsing the profiler's CSV files (trimmed real outputs under
tests/golden/rocprof/), the occupancy arithmetic, merging, and the best-so-far record."""
import json
import os

import pytest

from paper_2511_06345_amd import build, profile

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "rocprof")
MFMA = "void pgk::gemm_mfma_kernel<pgk::MfmaCfg<true, 256, 256, 64, 4, 2, 3, 2> >(pgk::GemmArgs, int)"


def test_default_groups_fit_the_hardware():
    raw_per_group = {"sq": 5, "fetch": 3, "write": 2, "l2": 2}       # raw counters behind each group
    assert [g for g, _ in profile.DEFAULT_GROUPS] == list(raw_per_group)
    assert raw_per_group["sq"] <= profile.BLOCK_LIMIT["SQ"]
    assert max(raw_per_group["fetch"], raw_per_group["write"], raw_per_group["l2"]) <= profile.BLOCK_LIMIT["TCC"]


def test_extra_counters_are_packed_within_block_limits():
    sq = [f"SQ_C{i}" for i in range(11)]
    passes = profile.plan_extra_passes(sq + ["TA_A", "TA_B", "TA_C", "TCC_X_sum", "TCC_X_max", "MyDerived", "SQ_C0"])
    for p in passes:
        per_block = {}
        for name in p:
            blk = profile.counter_block(name)
            if blk is None:
                assert p == [name]                      # a derived metric runs alone
                continue
            per_block.setdefault(blk, set()).add(profile._base(name))
        for blk, names in per_block.items():
            assert len(names) <= profile.BLOCK_LIMIT[blk]
    flat = [n for p in passes for n in p]
    assert sorted(flat) == sorted(set(sq + ["TA_A", "TA_B", "TA_C", "TCC_X_sum", "TCC_X_max", "MyDerived"]))
    assert len([p for p in passes if any(n.startswith("SQ_") for n in p)]) == 2     # 11 SQ counters: 8 + 3
    # the _sum and _max forms of one counter share a slot
    assert any("TCC_X_sum" in p and "TCC_X_max" in p for p in passes)
    assert profile.plan_extra_passes([]) == []


def test_kernel_trace_is_parsed_per_kernel():
    t = profile.parse_kernel_trace(os.path.join(GOLD, "c4_kernel_trace.csv"))
    assert set(t) == {"__amd_rocclr_copyBuffer", MFMA, "pgk::rowsum_combine_kernel(float const*, float*, int, int, int)"}
    m = t[MFMA]
    assert m["calls"] == 4 and m["workgroup_size"] == 512 and m["grid_size"] == 131072
    assert m["lds_bytes_per_workgroup"] == 163840 and m["scratch_bytes_per_lane"] == 0
    durations = [18813551057 - 18813432552, 18814046235 - 18813931689, 18814162821 - 18814050955, 18814279526 - 18814167540]
    assert m["avg_ns"] == sum(durations) / 4 and m["min_ns"] == min(durations) and m["max_ns"] == max(durations)
    # the first dispatch of each kernel dropped as warm-up
    t1 = profile.parse_kernel_trace(os.path.join(GOLD, "c4_kernel_trace.csv"), warmup_calls=1)
    assert t1[MFMA]["calls"] == 3 and t1[MFMA]["avg_ns"] == sum(durations[1:]) / 3
    assert t1["__amd_rocclr_copyBuffer"]["calls"] == 1      # never dropped to nothing


def test_counters_and_copy_calibration():
    c = profile.parse_counters(os.path.join(GOLD, "c3_fetch_counter_collection.csv"))
    assert list(c) == [MFMA]
    assert c[MFMA]["FETCH_SIZE"] == pytest.approx((786820.125 + 786866.8125 + 786985.0) / 3, rel=1e-4)
    cal = profile.parse_counters(os.path.join(GOLD, "cal_fetch_counter_collection.csv"))
    scale = profile.copy_scale(cal, "FETCH_SIZE", float(1 << 30))
    assert scale == pytest.approx(2.0, rel=1e-4)             # the counter sees half of a copy's bytes
    assert profile.copy_scale(cal, "WRITE_SIZE", float(1 << 30)) is None


def test_occupancy_arithmetic():
    # the large bf16 tile: 223 registers -> 224 allocated -> 2 waves; 160 KiB LDS -> one workgroup of 8 waves -> 2
    assert profile.occupancy_limits(223, 163840, 512) == {"by_registers": 2, "by_lds": 2, "waves_per_simd": 2, "max_waves_per_simd": 8}
    assert profile.occupancy_limits(20, 0, 256)["waves_per_simd"] == 8
    assert profile.occupancy_limits(128, 81920, 256) == {"by_registers": 4, "by_lds": 2, "waves_per_simd": 2, "max_waves_per_simd": 8}
    assert profile.occupancy_limits(184, 66560, 256)["by_registers"] == 2
    assert profile.occupancy_limits(300, 0, 64)["by_registers"] == 1


def test_merge_fills_the_metric_set():
    trace = profile.parse_kernel_trace(os.path.join(GOLD, "c4_kernel_trace.csv"))
    counters = {MFMA: {"FETCH_SIZE": 1000.0, "WRITE_SIZE": 500.0, "MfmaUtil": 61.0, "OccupancyPercent": 24.0,
                       "LdsUtil": 40.0, "LDSBankConflict": 0.0, "VALUBusy": 3.0, "TCC_HIT_sum": 81.0, "TCC_MISS_sum": 19.0,
                       "SQ_INSTS_LDS": 123.0}}
    resources = {"void pgk::gemm_mfma_kernel<pgk::MfmaCfg<true, 256, 256, 64, 4, 2, 3, 2>>(pgk::GemmArgs, int)":
                 {"vgprs": 223, "agprs": 0, "sgprs": 106, "scratch_bytes_per_lane": 0, "vgpr_spills": 0, "sgpr_spills": 20,
                  "lds_bytes_per_workgroup": 163840, "waves_per_simd": 2}}
    out = profile.merge(trace, counters, resources, fetch_scale=2.0, write_scale=1.0)
    assert [k["kernel"] for k in out] == [MFMA, "pgk::rowsum_combine_kernel(float const*, float*, int, int, int)"]
    k = out[0]
    assert k["registers"]["vgprs"] == 223 and k["registers"]["source"] == "compiler"     # matched despite "> >" vs ">>"
    assert k["lds"]["fraction_of_cu"] == 1.0 and k["occupancy"]["waves_per_simd"] == 2
    assert k["matrix_unit_busy_percent"] == 61.0 and k["occupancy"]["measured_percent"] == 24.0
    assert k["memory"]["read_bytes"] == 1000 * 1024 * 2.0 and k["memory"]["written_bytes"] == 500 * 1024
    assert k["memory"]["gb_per_s"] == pytest.approx((2048000 + 512000) / trace[MFMA]["avg_ns"])
    assert k["memory"]["l2_hit_percent"] == 81.0
    assert k["extra_counters"] == {"SQ_INSTS_LDS": 123.0}
    assert out[1]["registers"]["source"] == "kernel trace" and out[1]["workgroups"] == 64
    assert len(profile.merge(trace, counters, resources, 2.0, 1.0, all_kernels=True)) == 3


def test_markdown_summary_names_the_command_and_every_kernel():
    trace = profile.parse_kernel_trace(os.path.join(GOLD, "c4_kernel_trace.csv"))
    kernels = profile.merge(trace, {MFMA: {"FETCH_SIZE": 1000.0, "WRITE_SIZE": 500.0, "MfmaUtil": 61.0}}, {}, 2.0, 1.0)
    prof = {"workload": "c4", "step_time_us": 120.0, "kernels": kernels,
            "counter_scale": {"FETCH_SIZE": 2.0, "WRITE_SIZE": 1.0, "source": "test"}}
    text = profile.to_markdown(prof, "python3 bench.py --profile --workload c4")
    assert "python3 bench.py --profile --workload c4" in text and "MfmaUtil" in text
    assert text.count("## `") == 2 and "61.0 %" in text and "FETCH_SIZE x 2.0000" in text


def test_best_so_far_record(tmp_path):
    path = str(tmp_path / "best.json")
    a = {"workload": "c3", "when": "t0", "step_time_us": 900.0, "kernels": [{"kernel": "k", "time_us": 900.0}]}
    v = profile.update_record(path, "c3", a)
    assert v["is_new_best"] and v["previous_best_us"] is None
    slower = dict(a, step_time_us=990.0, when="t1")
    v = profile.update_record(path, "c3", slower)
    assert not v["is_new_best"] and v["change_percent"] == pytest.approx(10.0) and v["best_kernels"] == a["kernels"]
    assert json.load(open(path))["c3"]["when"] == "t0"            # the best is kept
    faster = dict(a, step_time_us=810.0, when="t2")
    v = profile.update_record(path, "c3", faster)
    assert v["is_new_best"] and v["change_percent"] == pytest.approx(-10.0)
    assert json.load(open(path))["c3"]["when"] == "t2"
    profile.update_record(path, "c4", dict(a, workload="c4"))
    assert set(json.load(open(path))) == {"c3", "c4"}


def test_compiler_remarks_are_parsed():
    text = """
x.hip:17:1: remark: Function Name: _ZN3pgk1aEv [-Rpass-analysis=kernel-resource-usage]
x.hip:17:1: remark:     TotalSGPRs: 25 [-Rpass-analysis=kernel-resource-usage]
x.hip:17:1: remark:     VGPRs: 10 [-Rpass-analysis=kernel-resource-usage]
x.hip:17:1: remark:     AGPRs: 4 [-Rpass-analysis=kernel-resource-usage]
x.hip:17:1: remark:     ScratchSize [bytes/lane]: 16 [-Rpass-analysis=kernel-resource-usage]
x.hip:17:1: remark:     Dynamic Stack: False [-Rpass-analysis=kernel-resource-usage]
x.hip:17:1: remark:     Occupancy [waves/SIMD]: 8 [-Rpass-analysis=kernel-resource-usage]
x.hip:17:1: remark:     SGPRs Spill: 1 [-Rpass-analysis=kernel-resource-usage]
x.hip:17:1: remark:     VGPRs Spill: 2 [-Rpass-analysis=kernel-resource-usage]
x.hip:17:1: remark:     LDS Size [bytes/block]: 4096 [-Rpass-analysis=kernel-resource-usage]
x.hip:40:1: remark: Function Name: _ZN3pgk1bEv [-Rpass-analysis=kernel-resource-usage]
x.hip:40:1: remark:     VGPRs: 99 [-Rpass-analysis=kernel-resource-usage]
"""
    r = build.parse_resource_remarks(text)
    assert r["_ZN3pgk1aEv"] == {"sgprs": 25, "vgprs": 10, "agprs": 4, "scratch_bytes_per_lane": 16, "waves_per_simd": 8,
                                "sgpr_spills": 1, "vgpr_spills": 2, "lds_bytes_per_workgroup": 4096}
    assert r["_ZN3pgk1bEv"] == {"vgprs": 99}


def test_built_library_comes_with_its_resource_table():
    if not os.path.exists(profile.RESOURCES):
        build.build_library()
    table = profile.load_resources()
    # (the shipping instance for plain GEMM operands: view 0, not the timed one)
    big = profile.match_resources(MFMA.replace("> >(", ">, 0, false>("), table)
    assert big is not None and big["scratch_bytes_per_lane"] == 0 and big["vgpr_spills"] == 0
    assert big["sgpr_spills"] <= 16
    assert big["lds_bytes_per_workgroup"] == 160 * 1024 and big["vgprs"] + big["agprs"] <= 256


def test_traffic_records_round_trip(tmp_path):
    """What the harness writes into a summary, bench.py reads back -- but only for the kernel
    sources the counters were taken with."""
    now = profile.kernel_source_hash()
    assert len(now) == 16 and now == profile.kernel_source_hash()
    kern = "void pgk::gemm_mfma_kernel<pgk::MfmaCfg<true, 256, 256, 64, 4, 2, 3, 2>, 0, false>(pgk::GemmArgs, int)"
    text = "\n".join(["# a summary", "`" + profile.traffic_record_line("c3", now, 1745802240.4, kern) + "`",
                      "`" + profile.traffic_record_line("c4", "0123456789abcdef", 235868169, kern) + "`", ""])
    (tmp_path / "x_metric_set.md").write_text(text)
    recs = profile.read_traffic_records(str(tmp_path))
    assert [r["workload"] for r in recs] == ["c3", "c4"] and recs[0]["bytes"] == 1745802240 and recs[0]["kernel"] == kern
    assert profile.stored_traffic("c3", "MfmaCfg<true, 256, 256, 64, 4, 2, 3, 2>, 0, false>", str(tmp_path)) == 1745802240
    assert profile.stored_traffic("c3", "MfmaCfg<true,256,256,64,4,2,3,2>,0,false>", str(tmp_path)) == 1745802240   # white space
    assert profile.stored_traffic("c4", "MfmaCfg<true, 256, 256, 64, 4, 2, 3, 2>, 0, false>", str(tmp_path)) is None  # other sources
    assert profile.stored_traffic("c3", "MfmaCfg<false, 128, 128", str(tmp_path)) is None
    assert profile.stored_traffic("c2", "MfmaCfg", str(tmp_path)) is None
