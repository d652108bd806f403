"""Pins for the adaptive-beta schedule (Eq. 3-4), the true-Nesterov extrapolation point (Eq. 10) and the
automatic fallback from "true" to "approx" after n_taylor steps."""
import math

import numpy as np
import pytest

from oracle import novak_oracle as O


def _h(**kw):
    base = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, rectified=False, nesterov="none", lookahead="none")
    base.update(kw)
    return O.Hyper(**base)


def test_schedule_values_and_limits():
    h = _h(adaptive_beta=True)
    b1, b2 = O.scheduled_betas(h, 1000)
    assert b1 == pytest.approx(0.9 * (1 - math.exp(-1.0)), rel=1e-15)         # t = tau_1
    assert b2 == pytest.approx(0.999 * (1 - math.exp(-0.2)), rel=1e-15)
    assert O.scheduled_betas(h, 10 ** 7) == pytest.approx((0.9, 0.999), rel=1e-12)   # asymptote: the base values
    prev = (0.0, 0.0)
    for t in range(1, 3000, 37):                                                # strictly increasing, below base
        cur = O.scheduled_betas(h, t)
        assert prev[0] < cur[0] < 0.9 and prev[1] < cur[1] < 0.999
        prev = cur
    assert O.scheduled_betas(_h(), 5) == (0.9, 0.999)
    assert O.scheduled_betas(_h(adaptive_beta=True, beta_tau1=10.0, beta_tau2=20.0), 10)[0] == pytest.approx(0.9 * (1 - math.exp(-1)))


def test_adaptive_beta_first_step_closed_form():
    """t = 1: beta1(1) ~ 9e-4, so m_1 = (1-beta1(1)) g; bias correction still divides by 1-beta1 (base)."""
    g = np.array([0.5, -2.0, 1e-3])
    h = _h(adaptive_beta=True)
    st = O.run([np.zeros(3)], lambda t: [g], 1, h, state_dtype=np.float64)[0]
    b1, b2 = 0.9 * (1 - math.exp(-1 / 1000)), 0.999 * (1 - math.exp(-1 / 5000))
    np.testing.assert_allclose(st.m, (1 - b1) * g, rtol=1e-14)
    np.testing.assert_allclose(st.v, (1 - b2) * g * g, rtol=1e-14)
    m_hat, v_hat = st.m / (1 - 0.9), st.v / (1 - 0.999)
    np.testing.assert_allclose(st.theta, -1e-3 * m_hat / (np.sqrt(v_hat) + 1e-8), rtol=1e-13)


def test_adaptive_beta_constant_gradient_recursion():
    """g = c: m_t = b_t m_{t-1} + (1-b_t) c with the scheduled b_t, unrolled independently."""
    c = 0.25
    h = _h(adaptive_beta=True, beta_tau1=7.0, beta_tau2=11.0)
    st = O.run([np.zeros(1)], lambda t: [np.array([c])], 30, h, state_dtype=np.float64)[0]
    m = v = 0.0
    for t in range(1, 31):
        b1 = 0.9 * (1 - math.exp(-t / 7.0))
        b2 = 0.999 * (1 - math.exp(-t / 11.0))
        m = b1 * m + (1 - b1) * c
        v = b2 * v + (1 - b2) * c * c
    assert st.m[0] == pytest.approx(m, rel=1e-14) and st.v[0] == pytest.approx(v, rel=1e-14)
    # m and v never exceed the gradient bound (Prop. 6.3 still holds; the schedule only tightens it)
    assert st.m[0] <= c and st.v[0] <= c * c


def test_extrapolation_point_sign_and_value():
    h = _h(beta_n=0.8)
    st = O.TensorState(np.array([1.0, -2.0], np.float32), np.array([0.5, 0.25], np.float32), np.zeros(2, np.float32))
    np.testing.assert_array_equal(O.extrapolate(st, h), np.array([1.0 + 0.8 * 0.5, -2.0 + 0.8 * 0.25]))


def test_true_nesterov_falls_back_to_approx_after_n_taylor():
    rng = np.random.default_rng(8)
    th = rng.normal(0, 0.02, 16)
    gs = [rng.normal(0, 1e-2, 16) for _ in range(8)]
    true3 = O.run([th], lambda t: [gs[t - 1]], 8, _h(nesterov="true", n_taylor=3), state_dtype=np.float64)[0]
    # the same thing by hand: steps 1-3 as "none" (the caller's gradient is used as is), steps 4-8 as "approx"
    st = O.init_state(th, _h(), np.float64)
    for t in range(1, 9):
        O.step(st, gs[t - 1], t, _h(nesterov="none" if t <= 3 else "approx"))
    np.testing.assert_array_equal(true3.theta, st.theta)
    assert [O.effective_nesterov(_h(nesterov="true", n_taylor=3), t) for t in (1, 3, 4, 9)] == ["true", "true", "approx", "approx"]
    assert O.effective_nesterov(_h(nesterov="true"), 10 ** 6) == "true"          # n_taylor = 0: never
    assert O.effective_nesterov(_h(nesterov="classical", n_taylor=3), 10) == "classical"
