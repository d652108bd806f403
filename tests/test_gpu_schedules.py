"""GPU parity of the adaptive-beta schedule (Eq. 3-4), the automatic true -> approx Nesterov fallback and
the extrapolation helper of Eq. 10."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import novak_oracle as O
from paper_2601_07876_amd import novak as N
from tests import harness as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nesterov,lookahead,grad_dtype,two_pass", [("approx", "memory_efficient", "f32", False),
                                                                    ("classical", "basic", "bf16", False),
                                                                    ("approx", "memory_efficient", "f32", True)])
def test_adaptive_beta(nesterov, lookahead, grad_dtype, two_pass):
    wl = W.get_workload("ragged")
    hyper = dict(wl.hyper, nesterov=nesterov, lookahead=lookahead, adaptive_beta=True, beta_tau1=4.0, beta_tau2=9.0,
                 layer_adaptation=two_pass)
    gpu, states, _ = H.run_pair(wl.numels, hyper, wl.steps, wl.grad_std, grad_dtype, auto_sync=True)
    try:
        H.compare_states(gpu, states)
    finally:
        gpu.close()
    # paper's time scales over 100 steps on the flat 2^18 prefix of configuration 1
    hyper = dict(W.get_workload("c1_flat_1m").hyper, adaptive_beta=True)
    gpu, states, _ = H.run_pair([1 << 18], hyper, 100, 1e-2, auto_sync=True)
    try:
        H.compare_states(gpu, states)
    finally:
        gpu.close()


@pytest.mark.parametrize("variant", ["single_pass", "device_step", "two_pass", "bf16_m"])
def test_adaptive_beta_keeps_a_small_second_moment_accurate(variant):
    """While beta_2(t) is near 0 (t << tau_2) the new v is ~beta_2(t) times the old one wherever the gradient has
    dropped; with gradients of order 1 that is far above the absolute floor of the bound, so v must be right in
    RELATIVE terms on every element (an evaluation that rounds at the old moment's magnitude is off by
    2^-24 / beta_2(t) ~ 1e-4 there)."""
    numels = [70001, 4097, 255, 1]
    # (no Nesterov term: the gradient that enters Eq. 2 is an input, so the EMA's own roundings are all there is)
    hyper = dict(W.get_workload("ragged").hyper, adaptive_beta=True, lookahead="none", nesterov="none", mode="research",
                 layer_adaptation=variant == "two_pass", moment_dtype="bf16_m" if variant == "bf16_m" else "f32",
                 device_step=variant == "device_step")
    steps = 6
    gpu, states, h = H.run_pair(numels, hyper, steps, 1.0, auto_sync=True, seed=7)
    try:
        H.compare_states(gpu, states, strict=False)
        b2 = O.scheduled_betas(h, steps)[1]
        assert b2 < 2e-3
        dropped = 0
        for got, st in zip(gpu.host("v"), states):
            ref = st.v.astype(np.float64)
            assert np.all(ref > 0.0)
            assert np.max(np.abs(got.astype(np.float64) - ref) / ref) < 1e-6
            dropped += int((ref < 4.0 * b2).sum())                     # v_t ~ beta_2(t) v_{t-1}: the gradient dropped
        assert dropped > 100
    finally:
        gpu.close()


def test_true_nesterov_fallback_after_n_taylor_steps():
    wl = W.get_workload("ragged")
    hyper = dict(wl.hyper, nesterov="true", n_taylor=4, mode="research")
    gpu, states, h = H.run_pair(wl.numels, hyper, 9, wl.grad_std)
    try:
        assert gpu.eff_nesterov == "true"
        H.compare_states(gpu, states)
    finally:
        gpu.close()
    # and it differs from never falling back
    a, _, _ = H.run_pair(wl.numels[:6], hyper, 9, wl.grad_std)
    b, _, _ = H.run_pair(wl.numels[:6], dict(hyper, n_taylor=0), 9, wl.grad_std)
    try:
        assert any(not np.array_equal(x, y) for x, y in zip(a.host("theta"), b.host("theta")))
    finally:
        a.close()
        b.close()


@pytest.mark.parametrize("misalign", [0, 1])
def test_extrapolation_point(misalign):
    """Eq. 10 after a few steps: out = theta + beta_n m, theta and m untouched, guards intact."""
    wl = W.get_workload("ragged")
    hyper = dict(wl.hyper, nesterov="true", mode="research", beta_n=0.7)
    gpu, states, h = H.run_pair(wl.numels, hyper, 4, wl.grad_std, misalign=misalign)
    try:
        outs_raw = [torch.full((n + 16,), -5.0, dtype=torch.float32, device="cuda:0") for n in wl.numels]
        outs = [r[4 + misalign: 4 + misalign + n] for r, n in zip(outs_raw, wl.numels)]
        th0, m0 = gpu.host("theta"), gpu.host("m")
        N.check(N.novak_nesterov_extrapolate(gpu.handle, [o.data_ptr() for o in outs], gpu.stream), "extrapolate", gpu.handle)
        torch.cuda.synchronize()
        for i, (o, st) in enumerate(zip(outs, states)):
            H.assert_close(f"extrapolated vs oracle state[{i}]", o.cpu().numpy(), O.extrapolate(st, h))
            # self-consistency with the state the library holds (a property, not an oracle input)
            own = th0[i].astype(np.float64) + 0.7 * m0[i].astype(np.float64)
            H.assert_close(f"extrapolated vs own state[{i}]", o.cpu().numpy(), own, atol=1e-9, rtol=2e-7)
            raw = outs_raw[i].cpu().numpy()
            assert np.all(raw[:4 + misalign] == -5.0) and np.all(raw[4 + misalign + wl.numels[i]:] == -5.0)
        for x, y in zip(th0, gpu.host("theta")):
            assert np.array_equal(x, y)
        assert N.novak_nesterov_extrapolate(gpu.handle, [0] * len(outs), gpu.stream) == N.NOVAK_ERR_NULL_POINTER
        assert N.novak_nesterov_extrapolate(gpu.handle, [o.data_ptr() + 2 for o in outs], gpu.stream) == N.NOVAK_ERR_MISALIGNED
    finally:
        gpu.close()


def test_back_to_back_extrapolations_with_different_output_lists():
    """Two calls in a row without a synchronisation in between: the second call's pointer list must not
    overtake the first call's kernel."""
    wl = W.get_workload("ragged")
    hyper = dict(wl.hyper, nesterov="true", mode="research", beta_n=0.7)
    gpu, states, h = H.run_pair(wl.numels, hyper, 3, wl.grad_std)
    try:
        a = [torch.full((n,), -5.0, dtype=torch.float32, device="cuda:0") for n in wl.numels]
        b = [torch.full((n,), -7.0, dtype=torch.float32, device="cuda:0") for n in wl.numels]
        torch.cuda.synchronize()
        for outs in (a, b, a):
            N.check(N.novak_nesterov_extrapolate(gpu.handle, [o.data_ptr() for o in outs], gpu.stream), "extrapolate", gpu.handle)
        torch.cuda.synchronize()
        for i, st in enumerate(states):
            ref = O.extrapolate(st, h)
            H.assert_close(f"a[{i}]", a[i].cpu().numpy(), ref)
            H.assert_close(f"b[{i}]", b[i].cpu().numpy(), ref)
    finally:
        gpu.close()
