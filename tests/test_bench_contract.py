"""Command-line contract of bench.py that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _run("--gpus", "2", "--steps", "1", "--warmup", "0")
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_variant_names_follow_the_lookahead_window():
    sys.path.insert(0, ROOT)
    import bench
    k = 5
    names = [bench.la_variant("memory_efficient", k, t, True) for t in range(1, 11)]
    assert names == ["step+la_first", "step+la_mid", "step+la_mid", "step+la_mid", "step+la_last_fused"] * 2
    assert [bench.la_variant("memory_efficient", k, t, False) for t in (5, 10)] == ["step+la_mid"] * 2
    assert [bench.la_variant("basic", k, t, True) for t in (1, 4, 5)] == ["step", "step", "step+basic_fused"]
    assert bench.la_variant("none", k, 5, True) == "step"
    assert bench.la_variant("memory_efficient", 1, 3, True) == "step+la_first"


def test_cpu_baseline_object_has_the_contract_keys():
    sys.path.insert(0, ROOT)
    import bench
    import workloads as W
    wl = W.get_workload("c2_resnet50")
    hyper = {k: v for k, v in wl.hyper.items()}
    out = bench.cpu_baseline(wl.name, hyper, 1 << 12, budget_s=0.2, max_steps=10)
    assert set(("value", "unit", "cores", "kind", "sample")) <= set(out)
    assert out["unit"] == "Gparams/s" and out["kind"] == "oracle" and out["cores"] == 1 and out["value"] > 0
