"""Where the direction of Eq. 17 is as steep as a decision, and what the comparison policy does about it (CPU).

While v_hat has no memory - the first step, or any early step under the adaptive-beta schedule of Eq. 3-4 - Eq. 17
is u = c1 g~ / (c2 |g~| + eps): a smoothed sign(g~) whose transition is ~eps wide.  If g~ is the small result of a
cancellation (g + lambda*theta with coupled decay, Eq. 13's g + beta_N (g - m)), an fp32 evaluation carries an
error of the size of the TERMS' roundings, and theta moves by far more than 1e-7 + 1e-5 |theta|.  The tests below
show the effect with the oracle alone, then run an fp32 evaluation of the step through the harness's CheckedOracle."""
import dataclasses

import numpy as np
import pytest

from oracle import novak_oracle as O
from tests import harness as H

f32 = np.float32


def test_first_step_direction_is_a_smoothed_sign_of_the_coupled_gradient():
    """Oracle alone: at t = 1, u = g~/(|g~| + eps) exactly (m_hat = g~, v_hat = g~^2), so a shift of the coupled
    gradient by 1e-11 - one fp32 rounding of lambda*theta - moves theta by lr * eps * 1e-11 / (|g~| + eps)^2."""
    h = O.Hyper(lr=1e-2, weight_decay=1e-2, decoupled_decay=False, rectified=False, nesterov="none", lookahead="none")
    theta = np.array([0.02, 0.02, 0.02])
    g_eff = np.array([1e-8, 1e-6, 1e-3])                   # what is left of g + lambda*theta
    g = g_eff - h.weight_decay * theta
    a = O.init_state(theta, h, np.float64)
    b = O.init_state(theta, h, np.float64)
    O.step(a, g, 1, h)
    O.step(b, g + 1e-11, 1, h)
    np.testing.assert_allclose(a.theta, theta - h.lr * g_eff / (np.abs(g_eff) + h.eps), rtol=1e-9)
    moved = np.abs(b.theta - a.theta)
    np.testing.assert_allclose(moved, h.lr * h.eps * 1e-11 / (np.abs(g_eff) + h.eps) ** 2, rtol=1e-3)
    bound = 1e-7 + 1e-5 * np.abs(a.theta)
    assert moved[0] > bound[0] and moved[1] < bound[1] and moved[2] < 1e-6 * bound[2]
    # the magnitudes of the terms, which is what an fp32 evaluation's error scales with, are in the trace
    np.testing.assert_allclose(a.trace.g_terms, np.abs(g) + h.weight_decay * np.abs(theta), rtol=1e-15)
    np.testing.assert_allclose(a.trace.g_processed, g_eff, rtol=1e-6)


def _fp32_first_step(theta, g, h):
    """Step 1 of the unrectified, coupled-decay configuration in fp32 (fused multiply-adds through double)."""
    def fma(a, b, c):
        return (np.asarray(a, np.float64) * np.float64(b) + np.asarray(c, np.float64)).astype(f32)
    s = O.step_scalars(h, 1)
    ge = fma(theta, f32(h.weight_decay), g)                                  # g + lambda*theta
    m = (f32(1.0 - h.beta1) * ge).astype(f32)                                # Eq. 1 from m_0 = 0
    v = (f32(1.0 - h.beta2) * (ge * ge).astype(f32)).astype(f32)             # Eq. 2 from v_0 = 0
    m_hat = (m * f32(1.0 / s.bc1)).astype(f32)
    v_hat = (v * f32(1.0 / s.bc2)).astype(f32)
    u = (m_hat / (np.sqrt(v_hat).astype(f32) + f32(h.eps))).astype(f32)      # Eq. 17
    th = (theta - (f32(s.step_size) * u).astype(f32)).astype(f32)            # Eq. 24, decay folded into g
    return th, m, v


def test_interval_policy_accepts_an_fp32_evaluation_and_nothing_wider():
    rng = np.random.default_rng(11)
    n = 1 << 14
    h = O.Hyper(lr=1e-2, weight_decay=1e-2, decoupled_decay=False, rectified=False, nesterov="none", lookahead="none")
    theta = rng.normal(0.0, 0.02, n).astype(f32)
    left = np.sign(rng.normal(size=n)) * 10.0 ** rng.uniform(-9.0, -5.0, n)   # what the cancellation leaves
    g = (left - h.weight_decay * theta.astype(np.float64)).astype(f32)
    th, m, v = _fp32_first_step(theta, g, h)

    def check(got_theta):
        states = [O.init_state(theta, h)]
        ck = H.CheckedOracle(states, h, "f32")
        ck.load([theta], [np.zeros(n, f32)], [np.zeros(n, f32)])
        ck.step([g], 1, [got_theta], [m], [v])
        return ck, states[0]

    ck, st = check(th)
    assert H.needs_common_state(h) and H.steep(h)
    # the situation exists: against the nominal result alone the fp32 evaluation is out of bounds somewhere ...
    nominal = O.init_state(theta, h)
    O.step(nominal, g, 1, h)
    outside = ~H._close(th, nominal.theta)
    assert 100 < outside.sum() < 0.5 * n                                      # (the input is made of cancellations)
    assert np.all(np.abs(nominal.trace.g_processed[outside]) < 1e-6)          # ... only where g + lambda*theta cancelled
    assert ck.in_interval == int(outside.sum())
    # ... and so frequent in this adversarial input that the rarity check refuses it
    with pytest.raises(AssertionError, match="interval"):
        ck.finish(1)
    # a result that is off by more than the interval allows is still refused, on a steep element or not
    j = int(np.argmax(outside))
    for k in (j, int(np.argmin(outside))):
        bad = th.copy()
        bad[k] += f32(1e-4)
        with pytest.raises(AssertionError, match="theta"):
            check(bad)


def test_interval_policy_survives_centralization():
    """The same with Eq. 26 in front on a tensor that is one row: a shift that every element shared would vanish
    with the row mean, so the policy shifts neighbouring elements in opposite directions."""
    rng = np.random.default_rng(12)
    n = 1 << 13
    h = O.Hyper(lr=1e-2, weight_decay=1e-2, decoupled_decay=False, rectified=False, nesterov="none", lookahead="none", use_gc=True)
    theta = rng.normal(0.0, 0.02, n).astype(f32)
    left = np.sign(rng.normal(size=n)) * 10.0 ** rng.uniform(-9.0, -5.0, n)
    c = left - h.weight_decay * theta.astype(np.float64)      # the centralized gradient that cancels against the decay
    c[-1] = -np.sum(c[:-1])                                   # a centralized row has mean 0
    g = (c + 3e-3).astype(f32)                                # the raw gradient: the same plus a row mean
    mean = float(np.mean(g.astype(np.float64)))
    gc = (g.astype(np.float64) - mean).astype(f32)            # Eq. 26 rounded once, then the step in fp32
    th, m, v = _fp32_first_step(theta, gc, dataclasses.replace(h, use_gc=False))

    states = [O.init_state(theta, h, rows=1)]
    ck = H.CheckedOracle(states, h, "f32")
    ck.load([theta], [np.zeros(n, f32)], [np.zeros(n, f32)])
    ck.step([g], 1, [th], [m], [v])
    nominal = O.init_state(theta, h, rows=1)
    O.step(nominal, g, 1, h)
    outside = ~H._close(th, nominal.theta)
    assert outside.sum() > 100 and ck.in_interval == int(outside.sum())
    # with one common shift for the whole row the interval collapses and the same evaluation is refused
    d_common = 1e-9
    a, b = O.init_state(theta, h, rows=1), O.init_state(theta, h, rows=1)
    O.step(a, g.astype(np.float64) + d_common, 1, h)
    O.step(b, g.astype(np.float64) - d_common, 1, h)
    assert np.max(np.abs(a.theta.astype(np.float64) - b.theta)) < 1e-7      # the shift dropped out with the mean


def test_which_runs_are_compared_step_by_step():
    base = dict(lookahead="none")
    assert not H.needs_common_state(O.Hyper(**base))
    assert not H.needs_common_state(O.Hyper(decoupled_decay=False, weight_decay=0.0, **base))   # nothing to couple
    assert H.needs_common_state(O.Hyper(decoupled_decay=False, weight_decay=1e-2, **base))
    assert H.needs_common_state(O.Hyper(adaptive_beta=True, **base))
    assert H.needs_common_state(O.Hyper(sparse_threshold=0.1, **base))
    assert H.needs_common_state(O.Hyper(moment_dtype="bf16_m", **base))
