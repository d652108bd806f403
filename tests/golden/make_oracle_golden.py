"""Writes tests/golden/oracle_c1_head.txt from the oracle alone (run from the repository root).

Configuration 1 of the benchmark (one flat fp32 tensor, fresh N(0,1e-2) gradients, 100 steps,
rectification + Nesterov approximation + memory-efficient lookahead k=5 alpha=0.5), restricted to
the first 4096 elements (the update is elementwise, so a prefix of the tensor is a valid run), under
both readings of the un-rectified phase.  The file stores the final theta, m, v of 16 elements as
hex floats; it guards the oracle against silent drift and is never written from GPU output.
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as W                      # noqa: E402
from oracle import novak_oracle as O       # noqa: E402

N, STEPS, PICK = 4096, 100, list(range(0, 4096, 256))


def compute(fallback):
    wl = W.get_workload("c1_flat_1m")
    hp = dict(wl.hyper)
    hp.pop("mode")
    hp["unrect_fallback"] = fallback
    h = O.Hyper(**hp)
    theta0 = [W.host_params([1 << 20], 42)[0][:N]]
    st = O.run(theta0, lambda t: [W.host_grads([1 << 20], t, wl.grad_std, 42)[0][:N]], STEPS, h)[0]
    return st


FULL_NUMELS, FULL_ROWS, FULL_STEPS = [48 * 64, 1000, 7], [48, 0, 0], 20


def compute_full(moment_dtype):
    """Every optional phase at once (research mode): clipping, centralization of the 48 x 64 tensor, scheduled
    betas, trust ratio, automatic rate, sparse mask, classical blend, lookahead; optionally a bfloat16 m."""
    h = O.Hyper(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=1e-2, beta_n=0.9, la_alpha=0.5, la_k=5,
                nesterov="classical", lookahead="memory_efficient", layer_adaptation=True, auto_lr=True,
                clip_threshold=0.4, sparse_threshold=0.3, use_gc=True, adaptive_beta=True, beta_tau1=30.0, beta_tau2=80.0,
                moment_dtype=moment_dtype)
    theta0 = W.host_params(FULL_NUMELS, 100)
    return O.run(theta0, lambda t: W.host_grads(FULL_NUMELS, t, 1e-2, 100), FULL_STEPS, h, rows=FULL_ROWS)


def write_full():
    lines = ["# written by tests/golden/make_oracle_golden.py from oracle/ only; hex floats (fp32 values)",
             "# moment_dtype tensor index theta m v"]
    for md in ("f32", "bf16_m"):
        for ti, st in enumerate(compute_full(md)):
            for i in range(0, st.theta.size, max(1, st.theta.size // 6)):
                lines.append(f"{md} {ti} {i} {float(st.theta[i]).hex()} {float(st.m[i]).hex()} {float(st.v[i]).hex()}")
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_full_features.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


def main():
    write_full()
    lines = ["# written by tests/golden/make_oracle_golden.py from oracle/ only; hex floats (fp32 values)",
             "# fallback index theta m v"]
    for fb in ("adam_denom", "sgdm"):
        st = compute(fb)
        for i in PICK:
            lines.append(f"{fb} {i} {float(st.theta[i]).hex()} {float(st.m[i]).hex()} {float(st.v[i]).hex()}")
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_c1_head.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
