"""Brute-force traces on 4-element tensors, in 60-digit decimal arithmetic, element by element.

An independent scalar walk through the ten phases (section 5.1, Table 2) for every combination of
the switches, 2k+1 steps so that two lookahead windows close and a third opens.  The walk below is
per element and per step, keeps every iterate of the window, and uses Python's `decimal` module
(no numpy, no shared helper with the oracle).  The oracle runs in all-double mode and must agree to
double rounding; a second check runs it with fp32 state and bounds the drift.
"""
import itertools
from decimal import Decimal, getcontext

import numpy as np
import pytest

from oracle import novak_oracle as O

getcontext().prec = 60
D = Decimal

K = 3
STEPS = 2 * K + 1
THETA0 = [0.25, -0.015625, 0.001953125, -3.0]
# gradients: exactly representable small numbers, a zero, sign flips, one large element
GRADS = [
    [0.0078125, -0.001953125, 0.0, 0.5],
    [-0.00390625, -0.0009765625, 0.000244140625, 0.25],
    [0.005859375, 0.001953125, -0.000244140625, -0.75],
    [0.0009765625, -0.0029296875, 0.0001220703125, 0.125],
    [-0.0068359375, 0.00048828125, 0.0, 0.375],
    [0.0029296875, -0.00146484375, -0.0003662109375, -0.0625],
    [0.001953125, 0.00244140625, 0.00006103515625, 0.4375],
]
HP = dict(lr="0.001", beta1="0.9", beta2="0.99", eps="0.00000001", wd="0.01", beta_n="0.8", la_alpha="0.5")


def _trace(rectified, decoupled, nesterov, lookahead, fallback, la_alpha=HP["la_alpha"]):
    lr, b1, b2, eps, wd, bn = (D(HP[k]) for k in ("lr", "beta1", "beta2", "eps", "wd", "beta_n"))
    la = D(la_alpha)
    out = []
    for e in range(4):
        th, m, v = D(THETA0[e]), D(0), D(0)
        slow0, window = th, []
        for t in range(1, STEPS + 1):
            g = D(GRADS[t - 1][e])
            # per-step scalars
            bc1 = 1 - b1 ** t
            bc2 = 1 - b2 ** t
            rho_inf = 2 / (1 - b2) - 1
            rho_t = rho_inf - 2 * t * b2 ** t / bc2
            r, denom = D(1), True
            if rectified:
                if rho_t >= 5:
                    r = ((rho_t - 4) * (rho_t - 2) * rho_inf / ((rho_inf - 4) * (rho_inf - 2) * rho_t)).sqrt()
                elif fallback == "sgdm":
                    denom = False
            # Phase 2
            if not decoupled:
                g = g + wd * th
            if nesterov == "approx":
                g = g + bn * (g - m)
            # Phase 4
            m = b1 * m + (1 - b1) * g
            v = b2 * v + (1 - b2) * g * g
            # Phases 5, 8
            mh = m / bc1
            u = mh / ((v / bc2).sqrt() + eps) if denom else mh
            if nesterov == "classical":
                u = b1 * mh + (1 - b1) * u
            # Phase 9
            if decoupled:
                th = th * (1 - lr * wd)
            th = th - lr * r * u
            # Phase 10
            if lookahead != "none":
                window.append(th)
                if t % K == 0:
                    if lookahead == "memory_efficient":
                        th = slow0 + la * sum(w - slow0 for w in window) / K
                    else:
                        th = slow0 + la * (window[-1] - slow0)
                    slow0, window = th, []
        out.append((float(th), float(m), float(v)))
    return out


COMBOS = list(itertools.product([False, True], [False, True], ["none", "approx", "classical", "true"],
                                ["none", "memory_efficient", "basic"], ["adam_denom", "sgdm"]))


@pytest.mark.parametrize("rectified,decoupled,nesterov,lookahead,fallback", COMBOS)
def test_trace_all_switches(rectified, decoupled, nesterov, lookahead, fallback):
    if not rectified and fallback == "sgdm":
        pytest.skip("fallback reading is only reachable with rectification on")
    h = O.Hyper(lr=float(HP["lr"]), beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.01, beta_n=0.8,
                la_alpha=0.5, la_k=K, rectified=rectified, decoupled_decay=decoupled, nesterov=nesterov,
                lookahead=lookahead, unrect_fallback=fallback)
    want = _trace(rectified, decoupled, "none" if nesterov == "true" else nesterov, lookahead, fallback)
    st = O.run([np.array(THETA0)], lambda t: [np.array(GRADS[t - 1])], STEPS, h, state_dtype=np.float64)[0]
    for e in range(4):
        th, m, v = want[e]
        assert st.theta[e] == pytest.approx(th, rel=1e-12, abs=1e-18)
        assert st.m[e] == pytest.approx(m, rel=1e-12, abs=1e-18)
        assert st.v[e] == pytest.approx(v, rel=1e-12, abs=1e-24)
    # fp32 state: same trajectory within the parity bound used against the GPU
    st32 = O.run([np.array(THETA0)], lambda t: [np.array(GRADS[t - 1])], STEPS, h, state_dtype=np.float32)[0]
    assert st32.theta.dtype == np.float32
    for e in range(4):
        assert abs(float(st32.theta[e]) - want[e][0]) <= 1e-7 + 1e-5 * abs(want[e][0])
        assert abs(float(st32.m[e]) - want[e][1]) <= 1e-7 + 1e-5 * abs(want[e][1])


def test_trace_window_open_after_last_step():
    """After 2k+1 steps one iterate sits in the open window and slow_0 is the second sync's result."""
    h = O.Hyper(lr=1e-3, beta1=0.9, beta2=0.99, weight_decay=0.01, beta_n=0.8, la_k=K, la_alpha=0.5)
    st = O.run([np.array(THETA0)], lambda t: [np.array(GRADS[t - 1])], STEPS, h, state_dtype=np.float64)[0]
    assert len(st.window) == 1 and np.array_equal(st.window[0], st.theta)
    st6 = O.run([np.array(THETA0)], lambda t: [np.array(GRADS[t - 1])], 2 * K, h, state_dtype=np.float64)[0]
    assert np.array_equal(st6.theta, st.slow0)


def test_trace_alpha_one_basic_equals_no_lookahead_trajectory():
    """alpha_LA = 1 with "basic": syncing is the identity, so the whole run equals lookahead off."""
    a = _trace(True, True, "approx", "basic", "adam_denom", la_alpha="1")
    b = _trace(True, True, "approx", "none", "adam_denom")
    assert a == b
