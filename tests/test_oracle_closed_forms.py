"""Closed-form pins for the oracle: trajectories whose value is known without running an optimizer.

Each case picks inputs for which Eq. 1-31 collapse to a formula (first step from zero moments,
constant gradient, zero gradient, arithmetic-progression windows for lookahead), and checks the
oracle in all-double mode against that formula.
"""
import math

import numpy as np
import pytest

from oracle import novak_oracle as O

THETA0 = np.array([0.3, -0.02, 2.5e-2, -7.0])
C = np.array([1e-2, -3e-3, 2.0, -1e-6])        # constant gradients, mixed sign / scale


def _run(h, grads_fn, steps, theta0=THETA0):
    return O.run([theta0], lambda t: [grads_fn(t)], steps, h, state_dtype=np.float64)[0]


def test_first_step_adam_denom_is_sign_step():
    """m0 = v0 = 0: m_hat = g~, v_hat = g~^2 => theta1 = theta0(1-a*l) - a*g~/(|g~|+eps); rho_1 = 1 < 5."""
    h = O.Hyper(lr=1e-3, weight_decay=1e-2, eps=1e-8, beta_n=0.9, nesterov="approx", lookahead="none",
                rectified=True, unrect_fallback="adam_denom")
    st = _run(h, lambda t: C, 1)
    gt = (1 + h.beta_n) * C                       # Eq. 13 with m0 = 0
    want = THETA0 * (1 - 1e-3 * 1e-2) - 1e-3 * gt / (np.abs(gt) + 1e-8)
    np.testing.assert_allclose(st.theta, want, rtol=1e-13)
    np.testing.assert_allclose(st.m, (1 - h.beta1) * gt, rtol=1e-13)
    np.testing.assert_allclose(st.v, (1 - h.beta2) * gt * gt, rtol=1e-12)


def test_first_step_sgdm_fallback_is_gradient_step():
    h = O.Hyper(lr=1e-3, weight_decay=1e-2, beta_n=0.9, nesterov="approx", lookahead="none",
                rectified=True, unrect_fallback="sgdm")
    st = _run(h, lambda t: C, 1)
    want = THETA0 * (1 - 1e-3 * 1e-2) - 1e-3 * (1 + h.beta_n) * C
    np.testing.assert_allclose(st.theta, want, rtol=1e-13)


@pytest.mark.parametrize("rectified", [False, True])
def test_constant_gradient_none_mode(rectified):
    """g = c, no Nesterov, no decay: m_hat = c and v_hat = c^2 at every t, so every step is
    alpha*r_t*c/(|c|+eps) and theta_T = theta_0 - alpha*c/(|c|+eps) * sum_t r_t."""
    h = O.Hyper(lr=1e-3, weight_decay=0.0, eps=1e-8, nesterov="none", lookahead="none",
                rectified=rectified, unrect_fallback="adam_denom")
    T = 100
    st = _run(h, lambda t: C, T)
    sum_r = sum(O.step_scalars(h, t).r_t for t in range(1, T + 1))
    if not rectified:
        assert sum_r == T
    want = THETA0 - 1e-3 * C / (np.abs(C) + 1e-8) * sum_r
    np.testing.assert_allclose(st.theta, want, rtol=1e-11)
    np.testing.assert_allclose(st.m, C * (1 - 0.9 ** T), rtol=1e-11)
    np.testing.assert_allclose(st.v, C * C * (1 - 0.999 ** T), rtol=1e-10)


def test_constant_gradient_classical_blend():
    """Eq. 16 with m_hat = c, u = c/(|c|+eps): u_nest = beta1*c + (1-beta1)*c/(|c|+eps)."""
    h = O.Hyper(lr=1e-3, weight_decay=0.0, eps=1e-8, beta1=0.9, nesterov="classical", lookahead="none",
                rectified=False)
    T = 25
    st = _run(h, lambda t: C, T)
    u_nest = 0.9 * C + 0.1 * C / (np.abs(C) + 1e-8)
    np.testing.assert_allclose(st.theta, THETA0 - 1e-3 * T * u_nest, rtol=1e-11)


def test_constant_gradient_approx_moments():
    """Eq. 13 under g = c: m_{t-1} = known => g~_t known; check m against the unrolled sum.

    m_t = sum_i beta1^(t-i) (1-beta1) g~_i with g~_i = c*(1+beta_n) - beta_n*m_{i-1}; the fixed
    point of the recursion is m = c (g~ = c), which the EMA must approach geometrically at rate
    beta1 - (1-beta1)*beta_n.
    """
    b1, bn = 0.9, 0.5
    h = O.Hyper(lr=1e-3, weight_decay=0.0, beta1=b1, beta_n=bn, nesterov="approx", lookahead="none",
                rectified=False)
    T = 60
    st = _run(h, lambda t: C, T)
    rate = b1 - (1 - b1) * bn                    # m_t - c = rate * (m_{t-1} - c)
    np.testing.assert_allclose(st.m, C * (1 - rate ** T), rtol=1e-11)


def test_zero_gradient_pure_decay_prop_6_5():
    """g = 0: m = v = 0, u = 0/(0+eps) = 0, theta_t = (1 - alpha*lambda)^t * theta_0."""
    for nest in ("none", "approx", "classical"):
        h = O.Hyper(lr=1e-2, weight_decay=0.1, nesterov=nest, lookahead="none", rectified=True)
        T = 37
        st = _run(h, lambda t: np.zeros(4), T)
        np.testing.assert_allclose(st.theta, THETA0 * (1 - 1e-2 * 0.1) ** T, rtol=1e-12)
        assert not st.m.any() and not st.v.any()


def test_decay_uses_base_lr_not_rectified_lr():
    """Eq. 18: the decay factor is 1 - alpha*lambda even when r_t << 1 (t = 6 has r_t ~ 0.026)."""
    h = O.Hyper(lr=1e-2, weight_decay=0.5, nesterov="none", lookahead="none", rectified=True)
    st = O.init_state(THETA0, h, np.float64)
    for t in range(1, 7):
        before = st.theta.copy()
        s = O.step(st, np.zeros(4), t, h)
        np.testing.assert_allclose(st.theta, before * (1 - 1e-2 * 0.5), rtol=1e-14)
    assert s.r_t < 0.05


# ------------------------------------------------------------------------------------------------
# lookahead
# ------------------------------------------------------------------------------------------------
def _ap_hyper(mode, alpha, k):
    # constant gradient, no rectification / decay / Nesterov: every fast step moves theta by -delta
    return O.Hyper(lr=1e-3, weight_decay=0.0, eps=1e-8, nesterov="none", rectified=False,
                   lookahead=mode, la_alpha=alpha, la_k=k)


def test_lookahead_arithmetic_progression_separates_readings():
    """Fast iterates slow0 - i*delta, i = 1..5, alpha_LA = 0.5.
    mean of all k iterates (Theorem 6.2):  slow0 - 1.5*delta      <- "memory_efficient"
    last iterate (standard Lookahead):     slow0 - 2.5*delta      <- "basic"
    (net displacement)/k:                  slow0 - 0.5*delta      (sign-fixed literal Eq. 29; not built)
    k-1 terms over k:                      slow0 - 1.0*delta      (Eq. 29's index range; not built)
    """
    delta = 1e-3 * C / (np.abs(C) + 1e-8)
    me = _run(_ap_hyper("memory_efficient", 0.5, 5), lambda t: C, 5)
    np.testing.assert_allclose(me.theta, THETA0 - 1.5 * delta, rtol=1e-12)
    ba = _run(_ap_hyper("basic", 0.5, 5), lambda t: C, 5)
    np.testing.assert_allclose(ba.theta, THETA0 - 2.5 * delta, rtol=1e-12)
    assert np.max(np.abs(me.theta - (THETA0 - 0.5 * delta))) > 1e-4
    assert np.max(np.abs(me.theta - (THETA0 - 1.0 * delta))) > 1e-4
    # second window starts from the synced point: slow0' = theta after sync
    me2 = _run(_ap_hyper("memory_efficient", 0.5, 5), lambda t: C, 10)
    np.testing.assert_allclose(me2.theta, THETA0 - 3.0 * delta, rtol=1e-12)
    # between syncs theta is the fast iterate
    me7 = _run(_ap_hyper("memory_efficient", 0.5, 5), lambda t: C, 7)
    np.testing.assert_allclose(me7.theta, THETA0 - (1.5 + 2) * delta, rtol=1e-12)


@pytest.mark.parametrize("k", [1, 2, 5])
def test_lookahead_alpha_one(k):
    """alpha_LA = 1: "basic" returns the fast weights bit for bit for every k; "memory_efficient"
    returns the mean of the window's k iterates, which is the fast weights only for k = 1."""
    rng = np.random.default_rng(5)
    grads = [rng.normal(0, 1e-2, 4) for _ in range(k)]
    common = dict(lr=1e-3, weight_decay=1e-2, nesterov="approx", rectified=True, la_alpha=1.0, la_k=k)
    fast = O.init_state(THETA0, O.Hyper(lookahead="none", **common), np.float32)
    iterates = []
    for t, g in enumerate(grads, 1):
        O.step(fast, g, t, O.Hyper(lookahead="none", **common))
        iterates.append(fast.theta.astype(np.float64))
    ba = O.run([THETA0], lambda t: [grads[t - 1]], k, O.Hyper(lookahead="basic", **common))[0]
    assert np.array_equal(ba.theta, fast.theta)
    me = O.run([THETA0], lambda t: [grads[t - 1]], k, O.Hyper(lookahead="memory_efficient", **common))[0]
    mean = np.mean(iterates, axis=0)
    np.testing.assert_allclose(me.theta.astype(np.float64), mean, rtol=2e-7)
    if k == 1:
        assert np.array_equal(me.theta, fast.theta)
    else:
        assert not np.array_equal(me.theta, fast.theta)


def test_lookahead_sync_leaves_moments_and_timing():
    h = O.Hyper(lookahead="memory_efficient", la_k=3, la_alpha=0.5, nesterov="none", rectified=False)
    assert [O.sync_due(t, h) for t in range(1, 8)] == [False, False, True, False, False, True, False]
    assert not O.sync_due(3, O.Hyper(lookahead="none", la_k=3))
    rng = np.random.default_rng(1)
    st = O.init_state(THETA0, h, np.float64)
    for t in (1, 2, 3):
        O.step(st, rng.normal(0, 1, 4), t, h)
    m, v = st.m.copy(), st.v.copy()
    O.lookahead_sync(st, h)
    assert np.array_equal(st.m, m) and np.array_equal(st.v, v)
    assert st.window == [] and np.array_equal(st.slow0, st.theta)


def test_blend_buffer_equals_sync_value_at_full_window():
    """The running blend (1-a)*slow0 + (a/k)*sum(theta_i) that the harness compares single-buffer
    implementations with is Eq. 30's right-hand side when i = k."""
    from tests.harness import blend_buffer
    h = O.Hyper(lookahead="memory_efficient", la_k=4, la_alpha=0.7, nesterov="approx", rectified=True)
    rng = np.random.default_rng(2)
    st = O.init_state(THETA0, h, np.float64)
    for t in range(1, 5):
        O.step(st, rng.normal(0, 1e-2, 4), t, h)
    blend = blend_buffer(st, h)
    O.lookahead_sync(st, h)
    np.testing.assert_allclose(st.theta, blend, rtol=1e-13)
