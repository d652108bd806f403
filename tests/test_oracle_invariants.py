"""Invariants of the update that hold for any input (Prop. 6.3, elementwise independence, resume)."""
import numpy as np
import pytest

import workloads as W
from oracle import novak_oracle as O


def _hyper(**kw):
    base = dict(W.BASE_HYPER)
    base.pop("mode")
    base.update(kw)
    return O.Hyper(**base)


def test_prop_6_3_moment_bounds():
    """|g| <= G elementwise  =>  |m_t| <= G and v_t <= G^2 for every t (nesterov none: g enters raw)."""
    G = 0.05
    rng = np.random.default_rng(42)
    h = _hyper(nesterov="none", lookahead="none")
    st = O.init_state(rng.normal(0, 0.02, 1000), h)
    for t in range(1, 201):
        g = np.clip(rng.normal(0, 0.05, 1000), -G, G)
        O.step(st, g, t, h)
        assert np.max(np.abs(st.m)) <= G * (1 + 1e-6)
        assert np.max(st.v) <= G * G * (1 + 1e-6) and np.min(st.v) >= 0.0


@pytest.mark.parametrize("nesterov,lookahead", [("approx", "memory_efficient"), ("classical", "basic")])
def test_elementwise_independence_under_permutation_and_resplit(nesterov, lookahead):
    wl = W.get_workload("ragged")
    numels = wl.numels[:9]
    h = _hyper(nesterov=nesterov, lookahead=lookahead, la_k=3)
    theta = W.host_params(numels, 42)
    steps = 7
    a = O.run(theta, lambda t: W.host_grads(numels, t, 1e-2, 42), steps, h)
    flat_a = np.concatenate([s.theta for s in a])
    # one flat tensor, permuted
    perm = np.random.default_rng(0).permutation(flat_a.size)
    th_flat = np.concatenate(theta)[perm]
    b = O.run([th_flat], lambda t: [np.concatenate(W.host_grads(numels, t, 1e-2, 42))[perm]], steps, h)[0]
    assert np.array_equal(b.theta, flat_a[perm])
    assert np.array_equal(b.m, np.concatenate([s.m for s in a])[perm])
    assert np.array_equal(b.v, np.concatenate([s.v for s in a])[perm])


def test_resume_equivalence():
    """The state is (theta, m, v, slow weights, t): stopping and continuing changes nothing."""
    numels = [1021, 64]
    h = _hyper(la_k=5)
    theta = W.host_params(numels, 100)
    gf = lambda t: W.host_grads(numels, t, 1e-2, 100)
    full = O.run(theta, gf, 20, h)
    half = O.run(theta, gf, 10, h)                     # 10 is a sync step: window closed
    cont = O.run(None, gf, 10, h, t0=10, states=half)
    for x, y in zip(full, cont):
        assert np.array_equal(x.theta, y.theta) and np.array_equal(x.m, y.m) and np.array_equal(x.v, y.v)


def test_fp32_state_stays_within_parity_bound_of_double_state():
    """fp32 storage drifts from the all-double run by far less than the 1e-5/1e-7 parity bound."""
    wl = W.get_workload("c1_flat_1m")
    n = [4096]
    h = _hyper()
    theta = W.host_params(n, 42)
    gf = lambda t: W.host_grads(n, t, wl.grad_std, 42)
    s32 = O.run(theta, gf, 100, h, state_dtype=np.float32)[0]
    s64 = O.run(theta, gf, 100, h, state_dtype=np.float64)[0]
    err = np.abs(s32.theta.astype(np.float64) - s64.theta)
    assert np.all(err <= 0.2 * (1e-7 + 1e-5 * np.abs(s64.theta)))


def test_nan_and_inf_propagate_without_trapping():
    h = _hyper(lookahead="none")
    st = O.init_state(np.array([0.1, 0.2, 0.3]), h)
    with np.errstate(all="ignore"):
        O.step(st, np.array([np.nan, np.inf, 1e-3]), 1, h)
    assert np.isnan(st.theta[0]) and np.isnan(st.theta[1]) and np.isfinite(st.theta[2])
