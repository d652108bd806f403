"""bench.py run in-process on a small workload: the JSON line carries the contract's keys and is self-consistent."""
import json
import sys

import pytest

pytestmark = pytest.mark.gpu

CONTRACT = ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
            "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline")


@pytest.mark.parametrize("extra", [[], ["--moment-dtype", "bf16_m", "--no-extras"], ["--layer-adaptation", "--clip", "1.0", "--no-extras"],
                                   ["--layout", "separate"], ["--layout", "torch_one"], ["--layout", "torch_pool"], ["--layout", "separate_contiguous"], ["--separate-sync"], ["--use-gc", "--clip", "1.0", "--no-extras"],
                                   ["--nesterov", "true", "--mode", "research", "--extrapolate", "--no-extras"],
                                   ["--device-step"], ["--device-step", "--graph-steps", "5"]])
def test_bench_line(monkeypatch, capsys, extra):
    import bench
    # one in-process oracle run, no worker processes: nothing is spawned from a process that holds the GPU
    argv = ["bench.py", "--workload", "c2_resnet50", "--steps", "10", "--warmup", "5", "--cpu-workers", "1", "--cpu-sample", "65536"] + extra
    monkeypatch.setattr(sys, "argv", argv)
    bench.main()
    lines = [l for l in capsys.readouterr().out.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in CONTRACT:
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 10 and d["warmup"] == 5 and d["higher_is_better"] is True
    assert d["unit"] == "Gparams/s" and d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "f32"
    cfg = d["config"]
    assert cfg["workload"] == "c2_resnet50" and cfg["params"] == 25557032 and "model" not in cfg
    assert d["value"] == pytest.approx(cfg["params"] / (d["ms_per_step"] * 1e-3) / 1e9, rel=1e-9)
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert r["frac"] == pytest.approx(r["achieved"] / r["peak"]) and 0.05 < r["frac"] < 1.0
    k = d["kernels"][r["kernel"]]
    assert r["achieved"] == pytest.approx(cfg["params"] * k["bytes_per_param"] / (k["avg_ms"] * 1e-3) / 1e9)
    assert r["algorithmic_bytes_per_launch"] == cfg["params"] * k["bytes_per_param"]
    if "--graph-steps" in extra:
        assert d["kernels"]["graph_of_5_steps"]["launches"] == 2 and cfg["step_count"] == "device" and r["traffic"] is None
    else:
        assert sum(v["launches"] for n, v in d["kernels"].items() if n not in ("lookahead_sync", "nesterov_extrapolate")) == 10
    if "--extrapolate" in extra:
        assert cfg["nesterov"] == "true" and d["kernels"]["nesterov_extrapolate"]["launches"] == 10
        assert d["kernels"]["nesterov_extrapolate"]["bytes_per_param"] == 12.0
    if "--separate-sync" in extra:
        assert d["kernels"]["lookahead_sync"]["launches"] == 2 and d["kernels"]["lookahead_sync"]["bytes_per_param"] == 8.0
        assert cfg["sync"] == "separate"
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["unit"] == "Gparams/s" and c["value"] > 0 and c["sample"]
    assert "cpu_baseline_all_cores" not in d
    if "--layout" not in extra:
        assert cfg["layout"] == "arena"
    else:
        assert cfg["layout"] == extra[1] and r["traffic"] is None        # counters were taken on the arena only
    if "--device-step" in extra:
        assert cfg["step_count"] == "device" and "other_layouts" not in d
    elif not extra:
        # beside the headline: the layouts a PyTorch caller has, and the sync as its own kernel, from the same process
        o = d["other_layouts"]
        assert set(o) == {"torch_one_allocation_planned_layout", "torch_five_separate_allocations",
                          "torch_five_allocations_in_a_mem_pool_fed_by_the_library"}
        for v in o.values():
            assert v["unit"] == "Gparams/s" and v["value"] > 0 and 0.05 < v["frac"] < 1.0
            assert v["value"] == pytest.approx(cfg["params"] / (v["ms_per_step"] * 1e-3) / 1e9, rel=1e-9)
        ss = d["separate_sync"]
        assert ss["value"] > 0 and ss["sync_kernel"]["launches"] == 2 and ss["sync_kernel"]["bytes_per_param"] == 8.0
    else:
        assert "other_layouts" not in d and "separate_sync" not in d


def test_host_cost_tool_runs_and_reports(tmp_path):
    """novak_hostcost (C++ over the C ABI, built by paper_2601_07876_amd.build): a child process, JSON on stdout."""
    import os
    import subprocess
    import workloads as W
    from paper_2601_07876_amd import build as B
    if not os.path.exists(B.HOSTCOST_PATH):          # normally built beforehand by `python -m paper_2601_07876_amd.build`
        B.build_hostcost(verbose=False)
    assert os.path.exists(B.HOSTCOST_PATH)
    f = tmp_path / "numels.txt"
    f.write_text("\n".join(str(n) for n in W.get_workload("ragged").numels) + "\n")
    out = subprocess.run([B.HOSTCOST_PATH, str(f), "200"], check=True, capture_output=True, text=True, timeout=120).stdout
    d = json.loads(out.strip().splitlines()[-1])
    assert d["tensors"] == len(W.get_workload("ragged").numels) and d["steps"] == 200
    assert 0.0 < d["host_us_per_step"] <= d["total_us_per_step"] < 1e4 and d["step_count"] == "host"
    # device-step mode, eager and as a captured graph of 10 steps replayed 20 times (the tool checks the device's count itself)
    out = subprocess.run([B.HOSTCOST_PATH, str(f), "200", "10"], check=True, capture_output=True, text=True, timeout=120).stdout
    d = json.loads(out.strip().splitlines()[-1])
    assert d["step_count"] == "device" and d["graph_steps"] == 10
    assert 0.0 < d["graph_host_us_per_step"] <= d["graph_us_per_step"] < 1e4 and 0.0 < d["total_us_per_step"] < 1e4
