"""Pins for the oracle's gradient clipping (sections 5.8, 7.3) and sparse threshold (Eq. 27)."""
import numpy as np
import pytest
import torch

from oracle import novak_oracle as O


def _h(**kw):
    base = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, rectified=False, nesterov="none",
                lookahead="none")
    base.update(kw)
    return O.Hyper(**base)


def test_clip_scale_closed_form_and_threshold():
    g = [np.array([3.0, 0.0]), np.array([0.0, 4.0, 0.0])]            # global norm 5
    assert O.clip_scale(g, _h(clip_threshold=1.0)) == pytest.approx(0.2, rel=1e-15)
    assert O.clip_scale(g, _h(clip_threshold=5.0)) == 1.0               # not above the threshold
    assert O.clip_scale(g, _h(clip_threshold=7.0)) == 1.0
    assert O.clip_scale(g, _h(clip_threshold=0.0)) == 1.0               # off
    scaled = [x * O.clip_scale(g, _h(clip_threshold=1.0)) for x in g]
    assert np.sqrt(sum(float(np.dot(x, x)) for x in scaled)) == pytest.approx(1.0, rel=1e-15)


def test_clip_matches_torch_clip_grad_norm():
    """torch.nn.utils.clip_grad_norm_ scales by max_norm/(norm + 1e-6): equal up to that 1e-6."""
    rng = np.random.default_rng(0)
    gs = [rng.normal(0, 1.0, 300), rng.normal(0, 2.0, 50)]
    ps = [torch.nn.Parameter(torch.zeros(len(g), dtype=torch.float64)) for g in gs]
    for p, g in zip(ps, gs):
        p.grad = torch.tensor(g)
    torch.nn.utils.clip_grad_norm_(ps, max_norm=1.0)
    s = O.clip_scale(gs, _h(clip_threshold=1.0))
    for p, g in zip(ps, gs):
        np.testing.assert_allclose(p.grad.numpy(), g * s, rtol=1e-6)


def test_clipping_is_global_and_precedes_everything_else():
    """Two tensors share one factor; with g' = s*g the whole step equals an unclipped step on g'."""
    rng = np.random.default_rng(1)
    th = [rng.normal(0, 0.02, 40), rng.normal(0, 0.02, 7)]
    gs = [[rng.normal(0, 3.0, 40), rng.normal(0, 0.1, 7)] for _ in range(6)]
    kw = dict(nesterov="approx", rectified=True, weight_decay=0.1, decoupled_decay=False, lookahead="memory_efficient", la_k=3)
    a = O.run(th, lambda t: gs[t - 1], 6, _h(clip_threshold=1.0, **kw), state_dtype=np.float64)
    pre = [[x * O.clip_scale(g, _h(clip_threshold=1.0)) for x in g] for g in gs]
    b = O.run(th, lambda t: pre[t - 1], 6, _h(**kw), state_dtype=np.float64)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x.theta, y.theta, rtol=1e-13)
        np.testing.assert_allclose(x.v, y.v, rtol=1e-13)
    # the factor really is below one for these gradients
    assert all(O.clip_scale(g, _h(clip_threshold=1.0)) < 0.2 for g in gs)


def test_sparse_threshold_first_step_closed_form():
    """t = 1 from zero moments: u = g/(|g|+eps); elements with |u| <= tau do not move (no decay)."""
    g = np.array([1e-9, -3e-9, 2e-8, -1.0, 0.0])
    u = g / (np.abs(g) + 1e-8)
    h = _h(sparse_threshold=0.5)
    st = O.run([np.ones(5)], lambda t: [g], 1, h, state_dtype=np.float64)[0]
    want = np.where(np.abs(u) > 0.5, 1.0 - 1e-3 * u, 1.0)
    np.testing.assert_allclose(st.theta, want, rtol=1e-15)
    assert list(np.abs(u) > 0.5) == [False, False, True, True, False]
    # moments are not masked
    np.testing.assert_allclose(st.m, 0.1 * g, rtol=1e-14)


def test_sparse_mask_comes_before_the_classical_blend_and_after_the_trust_ratio():
    g = np.array([1e-9, -1.0, 0.5, 2e-9])
    theta = np.array([1.0, 2.0, -1.0, 0.5])
    u = g / (np.abs(g) + 1e-8)
    masked = np.where(np.abs(u) > 0.5, u, 0.0)
    # classical: u_nest = beta1*m_hat + (1-beta1)*masked  (m_hat = g at t = 1)
    st = O.run([theta], lambda t: [g], 1, _h(sparse_threshold=0.5, nesterov="classical"), state_dtype=np.float64)[0]
    np.testing.assert_allclose(st.theta, theta - 1e-3 * (0.9 * g + 0.1 * masked), rtol=1e-14)
    # trust ratio uses the unmasked direction
    eta = np.linalg.norm(theta) / np.linalg.norm(u)
    st = O.run([theta], lambda t: [g], 1, _h(sparse_threshold=0.5, layer_adaptation=True), state_dtype=np.float64)[0]
    np.testing.assert_allclose(st.theta, theta - 1e-3 * eta * masked, rtol=1e-13)


def test_gradient_centralization_matches_library_definition():
    """Eq. 26 on a 4-D conv gradient: g - mean over dims 1..3, against torch's mean reduction."""
    rng = np.random.default_rng(3)
    shape = (6, 3, 5, 5)
    g = rng.normal(0.3, 1.0, shape)
    want = torch.tensor(g) - torch.tensor(g).mean(dim=(1, 2, 3), keepdim=True)
    h = _h(use_gc=True, lr=1.0, beta1=0.0, beta2=0.0, eps=1e-300)      # m = g_c after one step
    st = O.run([np.zeros(g.size)], lambda t: [g.reshape(-1)], 1, h, state_dtype=np.float64, rows=[6])[0]
    np.testing.assert_allclose(st.m, want.numpy().reshape(-1), rtol=1e-12, atol=1e-15)
    # each dim-0 slice of the centralized gradient sums to zero
    assert np.max(np.abs(st.m.reshape(6, -1).sum(axis=1))) < 1e-12
    # vectors (rows = 0) are left alone, and so is everything when use_gc is off
    st1 = O.run([np.zeros(g.size)], lambda t: [g.reshape(-1)], 1, h, state_dtype=np.float64, rows=[0])[0]
    np.testing.assert_allclose(st1.m, g.reshape(-1), rtol=1e-15)
    st2 = O.run([np.zeros(g.size)], lambda t: [g.reshape(-1)], 1, _h(lr=1.0, beta1=0.0, beta2=0.0), state_dtype=np.float64, rows=[6])[0]
    np.testing.assert_allclose(st2.m, g.reshape(-1), rtol=1e-15)


def test_centralization_order_after_clip_before_nesterov():
    """clip -> centralize -> approximation: equals feeding the pre-processed gradient to a plain run."""
    rng = np.random.default_rng(4)
    rows, cols = 5, 12
    th = [rng.normal(0, 0.02, rows * cols), rng.normal(0, 0.02, 9)]
    gs = [[rng.normal(0.5, 2.0, rows * cols), rng.normal(0, 2.0, 9)] for _ in range(5)]
    kw = dict(nesterov="approx", rectified=True, weight_decay=0.01)
    a = O.run(th, lambda t: gs[t - 1], 5, _h(clip_threshold=1.0, use_gc=True, **kw), state_dtype=np.float64, rows=[rows, 0])
    pre = []
    for g in gs:
        s = 1.0 / np.sqrt(sum(float(np.dot(x, x)) for x in g))       # all norms exceed 1
        g0 = (g[0] * s).reshape(rows, cols)
        pre.append([(g0 - g0.mean(axis=1, keepdims=True)).reshape(-1), g[1] * s])
    b = O.run(th, lambda t: pre[t - 1], 5, _h(**kw), state_dtype=np.float64)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x.theta, y.theta, rtol=1e-12)
        np.testing.assert_allclose(x.m, y.m, rtol=1e-11, atol=1e-18)


def test_centralization_degenerate_rows():
    """rows = numel: every slice is one element, the centralized gradient is zero; rows = 1: global mean."""
    g = np.array([1.0, 2.0, 4.0, 9.0])
    h = _h(use_gc=True, lr=1.0, beta1=0.0, beta2=0.0)
    st = O.run([np.zeros(4)], lambda t: [g], 1, h, state_dtype=np.float64, rows=[4])[0]
    assert not st.m.any()
    st = O.run([np.zeros(4)], lambda t: [g], 1, h, state_dtype=np.float64, rows=[1])[0]
    np.testing.assert_allclose(st.m, g - 4.0, rtol=1e-15)
