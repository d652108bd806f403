"""Seeded random combinations of every option of the step, on random ragged lists, against the oracle.

Each case draws a tensor list (sizes around the vector, wave, chunk and span boundaries, empty tensors included),
a hyper-parameter set (every Nesterov / lookahead / fallback / decay mode, clipping, centralization with random
row counts, sparse threshold, adaptive beta, trust ratio, automatic rate, bfloat16 first moment, device-step
mode), gradient type, misaligned views, chunk size and launch shape, runs 2k + 1..4 steps through the C ABI and
compares every element with the oracle under the harness's policy.  The seeds are fixed: the cases are the same
on every run."""
import random

import pytest

import workloads as W
from tests import harness as H

pytestmark = pytest.mark.gpu

SIZES = [0, 1, 2, 3, 5, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 4095, 4096, 4097, 16383, 16384, 16385, 20000, 70001, 131075]


def divisors(n):
    return [d for d in (1, 2, 3, 4, 5, 7, 8, 16, 64, 100, 256, 1000) if n % d == 0 and d <= n]


def draw_case(seed):
    rnd = random.Random(seed)
    base = dict(W.get_workload("ragged").hyper)
    numels = [rnd.choice(SIZES) if rnd.random() < 0.7 else rnd.randint(1, 90000) for _ in range(rnd.randint(1, 8))]
    k = rnd.choice([1, 2, 3, 5])
    hyper = dict(base, mode="research", nesterov=rnd.choice(["none", "approx", "classical", "true"]),
                 lookahead=rnd.choice(["none", "memory_efficient", "basic"]), la_k=k, la_alpha=rnd.choice([0.5, 0.8, 1.0]),
                 unrect_fallback=rnd.choice(["adam_denom", "sgdm"]), rectified=rnd.random() < 0.7,
                 decoupled_decay=rnd.random() < 0.7, weight_decay=rnd.choice([0.0, 1e-2]), lr=rnd.choice([1e-3, 1e-2]),
                 clip_threshold=rnd.choice([0.0, 0.0, 0.3]), sparse_threshold=rnd.choice([0.0, 0.0, 0.05]),
                 adaptive_beta=rnd.random() < 0.25, moment_dtype=rnd.choice(["f32", "f32", "bf16_m"]),
                 layer_adaptation=rnd.random() < 0.3, auto_lr=rnd.random() < 0.3, use_gc=rnd.random() < 0.3)
    if hyper["nesterov"] == "true":
        hyper["n_taylor"] = rnd.choice([0, 3])
    device_step = rnd.random() < 0.4
    if device_step:
        hyper["device_step"] = True
    rows = None
    if hyper["use_gc"]:
        rows = [rnd.choice(divisors(n)) if n > 0 and rnd.random() < 0.8 else 0 for n in numels]
    kw = dict(grad_dtype=rnd.choice(["f32", "bf16"]), seed=seed, auto_sync=True if device_step else rnd.random() < 0.5, guard=8,
              rows=rows, misalign=rnd.choice([0, 0, 1, 2, 3]), grad_misalign=rnd.choice([0, 0, 1, 3]),
              chunk_elems=rnd.choice([None, 4096, 65536]))
    steps = 2 * k + rnd.randint(1, 4)
    if not hyper["use_gc"] and hyper["moment_dtype"] == "f32" and not device_step and rnd.random() < 0.4:
        kw["vec_per_lane"] = rnd.choice([1, 2, 4])          # the other launch shapes of the plain fp32 kernel
        kw["threads"] = rnd.choice([64, 128, 256])
    if rnd.random() < 0.2:
        kw["nontemporal"] = False
    return numels, hyper, steps, kw


@pytest.mark.parametrize("first", range(0, 240, 30))
def test_random_option_combinations(first):
    for seed in range(first, first + 30):
        numels, hyper, steps, kw = draw_case(seed)
        print(f"seed {seed}: numels={numels} steps={steps} hyper={hyper} {kw}", flush=True)
        gpu, states, _ = H.run_pair(numels, hyper, steps, 1e-2, **kw)
        try:
            # (the scale-aware extra check is calibrated for steps of the default rate)
            H.compare_states(gpu, states, strict=(hyper["lr"] == 1e-3), tag=f"seed {seed}: ")
            assert gpu.guards_intact(), f"seed {seed}: a guard band was written"
        finally:
            gpu.close()


def draw_centralized_case(seed):
    """Larger centralized (and clipped) tensors whose rows cross vector, wave, span and chunk boundaries in every way."""
    rnd = random.Random(seed)
    base = dict(W.get_workload("ragged").hyper)
    numels, rows = [], []
    for _ in range(rnd.randint(1, 4)):
        cols = rnd.choice([1, 3, 17, 63, 64, 65, 255, 256, 257, 512, 1000, 2048, 4095, 4096, 4097, 8192, 25088, 50000, 100003])
        r = rnd.randint(1, max(1, min(3000, 3_000_000 // cols)))
        numels.append(r * cols)
        rows.append(r if rnd.random() < 0.85 else 0)
    k = rnd.choice([1, 2, 3])
    hyper = dict(base, mode="research", use_gc=True, clip_threshold=rnd.choice([0.0, 0.3]), la_k=k,
                 lookahead=rnd.choice(["none", "memory_efficient"]), moment_dtype=rnd.choice(["f32", "bf16_m"]),
                 layer_adaptation=rnd.random() < 0.3, device_step=rnd.random() < 0.3)
    kw = dict(grad_dtype=rnd.choice(["f32", "bf16"]), seed=seed, auto_sync=True, guard=8, rows=rows,
              grad_misalign=rnd.choice([0, 0, 1]), chunk_elems=rnd.choice([None, 4096, 65536, 1 << 20]))
    return numels, hyper, k + 2, kw


@pytest.mark.parametrize("first", range(0, 30, 10))
def test_random_centralized_shapes(first):
    for seed in range(first, first + 10):
        numels, hyper, steps, kw = draw_centralized_case(seed)
        print(f"seed {seed}: numels={numels} steps={steps} hyper={hyper} {kw}", flush=True)
        gpu, states, _ = H.run_pair(numels, hyper, steps, 1e-2, **kw)
        try:
            H.compare_states(gpu, states, tag=f"seed {seed}: ")
            assert gpu.guards_intact(), f"seed {seed}: a guard band was written"
        finally:
            gpu.close()


@pytest.mark.parametrize("first", range(1000, 1024, 8))
def test_random_long_horizons(first):
    """The option draws of test_random_option_combinations over 40-100 steps (many lookahead windows, the
    rectification switching on, the schedules of Eq. 3-4 moving), tensors capped at 30000 elements."""
    for seed in range(first, first + 8):
        numels, hyper, _, kw = draw_case(seed)
        steps = random.Random(seed * 7 + 1).randint(40, 100)
        numels = [min(n, 30000) for n in numels]
        if kw.get("rows"):
            kw["rows"] = [r if (n and r and n % r == 0) else 0 for n, r in zip(numels, kw["rows"])]
        print(f"seed {seed}: numels={numels} steps={steps} hyper={hyper} {kw}", flush=True)
        gpu, states, _ = H.run_pair(numels, hyper, steps, 1e-2, **kw)
        try:
            H.compare_states(gpu, states, strict=False, tag=f"seed {seed}: ")
            assert gpu.guards_intact(), f"seed {seed}: a guard band was written"
        finally:
            gpu.close()
