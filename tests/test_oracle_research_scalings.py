"""Pins for the two full-features scalings of the oracle: the layer-wise trust ratio (Eq. 19, 25) and
the auto-LR factor (Eq. 20-22), and how they enter alpha_eff (Eq. 24a).

Closed forms on inputs where the norms are known by construction, clip boundaries, the zero-norm
convention, and a 60-digit decimal brute force over two tensors with both features on together with
rectification, Nesterov approximation and lookahead.
"""
from decimal import Decimal, getcontext

import numpy as np
import pytest

from oracle import novak_oracle as O

getcontext().prec = 60
D = Decimal


def _h(**kw):
    base = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, beta_n=0.9, rectified=False,
                nesterov="none", lookahead="none")
    base.update(kw)
    return O.Hyper(**base)


def test_trust_ratio_closed_form_first_step():
    """theta = a everywhere, g = c everywhere: u = c/(|c|+eps), ||theta||/||u|| = |a|(|c|+eps)/|c|,
    so theta_1 = a - alpha * |a| * sign(c) exactly (within the clip range)."""
    n, a, c = 1000, 0.5, -2e-3
    h = _h(layer_adaptation=True)
    st = O.run([np.full(n, a)], lambda t: [np.full(n, c)], 1, h, state_dtype=np.float64)[0]
    np.testing.assert_allclose(st.theta, a - 1e-3 * abs(a) * np.sign(c), rtol=1e-13)


@pytest.mark.parametrize("a,expected_eta", [(100.0, 10.0), (1e-3, 0.1), (3.0, 3.0)])
def test_trust_ratio_clip(a, expected_eta):
    n, c = 64, 1.0                       # u = 1/(1+eps) ~ 1, so eta ~ |a|
    h = _h(layer_adaptation=True)
    st = O.run([np.full(n, a)], lambda t: [np.full(n, c)], 1, h, state_dtype=np.float64)[0]
    np.testing.assert_allclose(a - st.theta, 1e-3 * expected_eta * (1.0 / (1.0 + 1e-8)) *
                               (1.0 if expected_eta in (10.0, 0.1) else (1.0 + 1e-8)), rtol=1e-12)


def test_trust_ratio_zero_norms_give_one():
    h = _h(layer_adaptation=True)
    assert O.trust_ratio(np.zeros(4), np.ones(4), h) == 1.0
    assert O.trust_ratio(np.ones(4), np.zeros(4), h) == 1.0
    # zero parameters: the step is the plain one
    a = O.run([np.zeros(8)], lambda t: [np.full(8, 0.3)], 1, h, state_dtype=np.float64)[0]
    b = O.run([np.zeros(8)], lambda t: [np.full(8, 0.3)], 1, _h(), state_dtype=np.float64)[0]
    assert np.array_equal(a.theta, b.theta)


def test_trust_ratio_is_per_tensor_and_uses_pre_blend_direction():
    """Two tensors with different scales get different ratios; classical blending does not change eta."""
    th = [np.full(16, 2.0), np.full(16, 0.5)]
    g = [np.full(16, 1e-2), np.full(16, -1e-2)]
    for nest in ("none", "classical"):
        h = _h(layer_adaptation=True, nesterov=nest)
        sts = O.run(th, lambda t: g, 1, h, state_dtype=np.float64)
        u = 1e-2 / (1e-2 + 1e-8)
        blend = (0.9 * 1e-2 + 0.1 * u) if nest == "classical" else u      # Eq. 16 with m_hat = g
        np.testing.assert_allclose(2.0 - sts[0].theta, 1e-3 * (2.0 / u) * blend, rtol=1e-12)
        np.testing.assert_allclose(sts[1].theta - 0.5, 1e-3 * (0.5 / u) * blend, rtol=1e-12)


def test_auto_lr_first_step_and_ema():
    """t = 1: g_bar/theta_bar = ||g||/||theta|| (gamma cancels); later steps follow Eq. 20-21."""
    th = [np.full(9, 1.0), np.full(16, 1.0)]                 # ||theta|| = 5
    g1 = [np.full(9, 0.5), np.full(16, 0.5)]                 # ||g|| = 2.5  -> ratio 0.5
    h = _h(auto_lr=True)
    aux = O.AutoLrState()
    states = [O.init_state(x, h, np.float64) for x in th]
    a1 = O.step_all(states, g1, 1, h, aux)
    assert a1 == pytest.approx(0.5, rel=1e-14)
    assert aux.g_bar == pytest.approx(0.25, rel=1e-14) and aux.theta_bar == pytest.approx(0.5, rel=1e-14)
    u = 0.5 / (0.5 + 1e-8)
    np.testing.assert_allclose(states[0].theta, 1.0 - 1e-3 * 0.5 * u, rtol=1e-13)
    # second step: EMAs mix in the new norms with weight gamma
    norm_theta2 = np.sqrt(sum(float(np.dot(s.theta, s.theta)) for s in states))
    g2 = [np.full(9, 2.0), np.full(16, 2.0)]                 # ||g|| = 10
    a2 = O.step_all(states, g2, 2, h, aux)
    assert aux.g_bar == pytest.approx(0.1 * 10.0 + 0.9 * 0.25, rel=1e-14)
    assert aux.theta_bar == pytest.approx(0.1 * norm_theta2 + 0.9 * 0.5, rel=1e-14)
    assert a2 == pytest.approx(aux.g_bar / aux.theta_bar, rel=1e-14)


@pytest.mark.parametrize("gscale,expected", [(100.0, 2.0), (1e-4, 0.1)])
def test_auto_lr_clip_and_zero_theta(gscale, expected):
    h = _h(auto_lr=True)
    aux = O.AutoLrState()
    states = [O.init_state(np.ones(4), h, np.float64)]
    assert O.step_all(states, [np.full(4, gscale)], 1, h, aux) == expected
    aux0 = O.AutoLrState()
    z = [O.init_state(np.zeros(4), h, np.float64)]
    assert O.step_all(z, [np.ones(4)], 1, h, aux0) == 1.0


def test_decay_is_not_scaled_by_trust_or_auto_lr():
    """Eq. 18 / 24: the decay term keeps the base alpha whatever lambda_trust and alpha_auto are."""
    h = _h(layer_adaptation=True, auto_lr=True, weight_decay=0.1)
    st = O.run([np.full(8, 50.0)], lambda t: [np.zeros(8)], 3, h, state_dtype=np.float64)[0]
    np.testing.assert_allclose(st.theta, 50.0 * (1 - 1e-3 * 0.1) ** 3, rtol=1e-13)


# ---- decimal brute force over two tensors, everything on ---------------------------------------------
THETA0 = [[0.25, -0.015625, 0.001953125, -3.0], [1.5, -0.75, 0.03125]]
GRADS = [
    [[0.0078125, -0.001953125, 0.0, 0.5], [0.25, -0.125, 0.0625]],
    [[-0.00390625, -0.0009765625, 0.000244140625, 0.25], [-0.5, 0.03125, 0.015625]],
    [[0.005859375, 0.001953125, -0.000244140625, -0.75], [0.125, 0.25, -0.0078125]],
    [[0.0009765625, -0.0029296875, 0.0001220703125, 0.125], [0.0625, -0.375, 0.5]],
    [[-0.0068359375, 0.00048828125, 0.0, 0.375], [-0.03125, 0.125, 0.25]],
    [[0.0029296875, -0.00146484375, -0.0003662109375, -0.0625], [0.75, 0.5, -0.125]],
    [[0.001953125, 0.00244140625, 0.00006103515625, 0.4375], [0.25, -0.0625, 0.375]],
]
K = 3


def _brute(layer, auto, nesterov):
    lr, b1, b2, eps, wd, bn, la, gam = D("0.001"), D("0.9"), D("0.99"), D("1e-8"), D("0.01"), D("0.8"), D("0.5"), D("0.1")
    th = [[D(x) for x in t] for t in THETA0]
    m = [[D(0)] * len(t) for t in THETA0]
    v = [[D(0)] * len(t) for t in THETA0]
    slow0 = [list(t) for t in th]
    window = [[] for _ in th]
    gbar = tbar = D(0)
    for t in range(1, 8):
        bc1, bc2 = 1 - b1 ** t, 1 - b2 ** t
        rho_inf = 2 / (1 - b2) - 1
        rho_t = rho_inf - 2 * t * b2 ** t / bc2
        r = ((rho_t - 4) * (rho_t - 2) * rho_inf / ((rho_inf - 4) * (rho_inf - 2) * rho_t)).sqrt() if rho_t >= 5 else D(1)
        a_auto = D(1)
        if auto:
            gn = sum(D(x) ** 2 for tens in GRADS[t - 1] for x in tens).sqrt()
            tn = sum(x ** 2 for tens in th for x in tens).sqrt()
            gbar = gam * gn + (1 - gam) * gbar
            tbar = gam * tn + (1 - gam) * tbar
            a_auto = min(max(gbar / tbar, D("0.1")), D(2))
        for i in range(len(th)):
            n = len(th[i])
            us, mh = [], []
            for e in range(n):
                g = D(GRADS[t - 1][i][e])
                if nesterov == "approx":
                    g = g + bn * (g - m[i][e])
                m[i][e] = b1 * m[i][e] + (1 - b1) * g
                v[i][e] = b2 * v[i][e] + (1 - b2) * g * g
                mh.append(m[i][e] / bc1)
                us.append(mh[e] / ((v[i][e] / bc2).sqrt() + eps))
            trust = D(1)
            if layer:
                nt = sum(x ** 2 for x in th[i]).sqrt()
                nu = sum(x ** 2 for x in us).sqrt()
                eta = nt / nu if (nt > 0 and nu > 0) else D(1)
                trust = min(max(eta, D("0.1")), D(10))
            for e in range(n):
                u = b1 * mh[e] + (1 - b1) * us[e] if nesterov == "classical" else us[e]
                th[i][e] = th[i][e] * (1 - lr * wd) - lr * r * trust * a_auto * u
            window[i].append(list(th[i]))
            if t % K == 0:
                for e in range(n):
                    th[i][e] = slow0[i][e] + la * sum(w[e] - slow0[i][e] for w in window[i]) / K
                slow0[i], window[i] = list(th[i]), []
    return [[float(x) for x in t] for t in th]


@pytest.mark.parametrize("layer,auto", [(True, False), (False, True), (True, True)])
@pytest.mark.parametrize("nesterov", ["approx", "classical"])
def test_brute_force_two_tensors(layer, auto, nesterov):
    h = O.Hyper(lr=1e-3, beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.01, beta_n=0.8, la_alpha=0.5, la_k=K,
                rectified=True, nesterov=nesterov, lookahead="memory_efficient", layer_adaptation=layer, auto_lr=auto)
    sts = O.run([np.array(t) for t in THETA0], lambda t: [np.array(g) for g in GRADS[t - 1]], 7, h,
                state_dtype=np.float64)
    want = _brute(layer, auto, nesterov)
    for st, w in zip(sts, want):
        np.testing.assert_allclose(st.theta, w, rtol=1e-11, atol=1e-18)
    # and the scalings really change the trajectory
    plain = O.run([np.array(t) for t in THETA0], lambda t: [np.array(g) for g in GRADS[t - 1]], 7,
                  O.Hyper(lr=1e-3, beta1=0.9, beta2=0.99, weight_decay=0.01, beta_n=0.8, la_k=K, nesterov=nesterov),
                  state_dtype=np.float64)
    assert max(np.max(np.abs(a.theta - b.theta)) for a, b in zip(sts, plain)) > 1e-5


def test_trace_holds_the_per_tensor_scale_and_the_steps_intermediates():
    """TensorState.trace after a step: lambda_trust * alpha_auto of Eq. 24a (what GPU tests compare the library's
    per-tensor scales with), and the intermediates the comparison policy reads - pinned here by closed forms at t = 1."""
    th = [np.full(4, 2.0), np.full(9, 0.5)]
    g = [np.full(4, 1e-2), np.full(9, 1e-2)]
    h = _h(layer_adaptation=True, auto_lr=True, trust_clip=(0.1, 1e3), auto_clip=(1e-6, 1e3))
    aux = O.AutoLrState()
    states = [O.init_state(x, h, np.float64) for x in th]
    a = O.step_all(states, g, 1, h, aux)
    u = 1e-2 / (1e-2 + 1e-8)                                  # m_hat = g, v_hat = g^2 at t = 1 (no Nesterov in _h)
    ratio = np.sqrt(13 * 1e-4) / np.sqrt(4 * 4.0 + 9 * 0.25)  # ||g|| / ||theta|| over both tensors
    assert a == pytest.approx(ratio, rel=1e-13)
    assert states[0].trace.scale == pytest.approx((2.0 / u) * ratio, rel=1e-13)     # eta = ||theta|| / ||u|| per tensor
    assert states[1].trace.scale == pytest.approx((0.5 / u) * ratio, rel=1e-13)
    tr = states[0].trace
    np.testing.assert_allclose(tr.u_base, u, rtol=1e-14)
    np.testing.assert_allclose(tr.m_exact, (1 - h.beta1) * 1e-2, rtol=1e-14)
    assert np.array_equal(tr.g_processed, tr.g_tilde) and np.array_equal(tr.g_tilde, np.full(4, 1e-2))
    # with the Nesterov approximation g_tilde = (1 + beta_n) g at t = 1 and g_processed stays the gradient handed in
    h2 = O.Hyper(lookahead="none", nesterov="approx", beta_n=0.7)
    st = O.init_state(np.ones(3), h2, np.float64)
    O.step(st, np.full(3, 0.2), 1, h2)
    np.testing.assert_allclose(st.trace.g_tilde, 1.7 * 0.2, rtol=1e-15)
    np.testing.assert_allclose(st.trace.g_processed, 0.2, rtol=1e-15)
    assert st.trace.scale == 1.0
