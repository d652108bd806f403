"""Special cases of the oracle that reduce to library optimizers (torch.optim on the CPU, fp64).

 * rectification, Nesterov and lookahead off  ->  AdamW (decoupled decay, Eq. 18) / Adam with L2
   (coupled reading), with epsilon added after the bias-corrected root (Eq. 17).
 * rectification on, "sgdm" fallback, Nesterov none, lookahead off  ->  RAdam with decoupled decay:
   same rho_t / r_t schedule (Eq. 6-9), momentum step while rho_t < 5.  torch's RAdam scales epsilon
   by 1/sqrt(1-beta2^t), so that comparison uses a vanishing epsilon.
 * rectification on, "adam_denom" fallback: the first five steps are AdamW steps (r_t = 1, Eq. 8).
"""
import numpy as np
import pytest
import torch

from oracle import novak_oracle as O

N = 257
STEPS = 40


def _inputs(seed=42, gstd=1e-2):
    rng = np.random.default_rng(seed)
    theta0 = rng.normal(0, 0.02, N)
    grads = [rng.normal(0, gstd, N) for _ in range(STEPS)]
    return theta0, grads


def _run_torch(opt_cls, theta0, grads, **kw):
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = opt_cls([p], foreach=False, **kw)
    traj = []
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        traj.append(p.detach().numpy().copy())
    st = opt.state[p]
    return traj, st["exp_avg"].numpy().copy(), st["exp_avg_sq"].numpy().copy()


def _run_oracle(theta0, grads, h):
    st = O.init_state(theta0, h, np.float64)
    traj = []
    for t, g in enumerate(grads, 1):
        O.step(st, g, t, h)
        if O.sync_due(t, h):
            O.lookahead_sync(st, h)
        traj.append(st.theta.copy())
    return traj, st.m, st.v


@pytest.mark.parametrize("wd", [0.0, 1e-2, 0.3])
def test_reduces_to_adamw(wd):
    theta0, grads = _inputs()
    h = O.Hyper(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=wd, rectified=False,
                nesterov="none", lookahead="none", decoupled_decay=True)
    ref, m, v = _run_torch(torch.optim.AdamW, theta0, grads, lr=1e-3, betas=(0.9, 0.999), eps=1e-8,
                           weight_decay=wd)
    got, gm, gv = _run_oracle(theta0, grads, h)
    for a, b in zip(got, ref):
        np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(gm, m, rtol=1e-12, atol=0)
    np.testing.assert_allclose(gv, v, rtol=1e-12, atol=0)


def test_reduces_to_adam_with_coupled_l2():
    theta0, grads = _inputs(seed=100)
    h = O.Hyper(lr=3e-3, beta1=0.8, beta2=0.99, eps=1e-8, weight_decay=0.1, rectified=False,
                nesterov="none", lookahead="none", decoupled_decay=False)
    ref, m, v = _run_torch(torch.optim.Adam, theta0, grads, lr=3e-3, betas=(0.8, 0.99), eps=1e-8,
                           weight_decay=0.1)
    got, gm, gv = _run_oracle(theta0, grads, h)
    for a, b in zip(got, ref):
        np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(gm, m, rtol=1e-12)
    np.testing.assert_allclose(gv, v, rtol=1e-12)


@pytest.mark.parametrize("beta2,wd", [(0.999, 0.0), (0.999, 1e-2), (0.99, 0.05), (0.95, 0.0)])
def test_reduces_to_radam_with_momentum_fallback(beta2, wd):
    theta0, grads = _inputs(seed=2025)
    tiny = 1e-100
    h = O.Hyper(lr=1e-3, beta1=0.9, beta2=beta2, eps=tiny, weight_decay=wd, rectified=True,
                nesterov="none", lookahead="none", unrect_fallback="sgdm")
    ref, m, v = _run_torch(torch.optim.RAdam, theta0, grads, lr=1e-3, betas=(0.9, beta2), eps=tiny,
                           weight_decay=wd, decoupled_weight_decay=True)
    got, gm, gv = _run_oracle(theta0, grads, h)
    for t, (a, b) in enumerate(zip(got, ref), 1):
        np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-15, err_msg=f"step {t}")
    np.testing.assert_allclose(gm, m, rtol=1e-12)
    np.testing.assert_allclose(gv, v, rtol=1e-12)


def test_adam_denom_fallback_takes_adamw_steps_until_rectified():
    theta0, grads = _inputs(seed=7)
    base = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=1e-2, nesterov="none",
                lookahead="none")
    rect, _, _ = _run_oracle(theta0, grads, O.Hyper(rectified=True, unrect_fallback="adam_denom", **base))
    ref, _, _ = _run_torch(torch.optim.AdamW, theta0, grads, lr=1e-3, betas=(0.9, 0.999), eps=1e-8,
                           weight_decay=1e-2)
    for t in range(5):
        np.testing.assert_allclose(rect[t], ref[t], rtol=1e-11, atol=1e-15)
    # from step 6 on r_t < 1 shortens the step: the two trajectories separate
    assert np.max(np.abs(rect[5] - ref[5])) > 1e-4
    # and "sgdm" differs from "adam_denom" already at step 1 (alpha*g vs alpha*sign(g))
    sg, _, _ = _run_oracle(theta0, grads, O.Hyper(rectified=True, unrect_fallback="sgdm", **base))
    assert np.max(np.abs(sg[0] - rect[0])) > 1e-4


def test_rectified_tail_equals_adamw_step_scaled_by_r_t():
    """With identical incoming state, a rectified step is the AdamW displacement times r_t."""
    theta0, grads = _inputs(seed=11)
    hb = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, nesterov="none", lookahead="none")
    h_r = O.Hyper(rectified=True, **hb)
    h_a = O.Hyper(rectified=False, **hb)
    st = O.init_state(theta0, h_r, np.float64)
    for t, g in enumerate(grads, 1):
        st_a = O.TensorState(st.theta.copy(), st.m.copy(), st.v.copy())
        before = st.theta.copy()
        s = O.step(st, g, t, h_r)
        O.step(st_a, g, t, h_a)
        np.testing.assert_allclose(st.theta - before, s.r_t * (st_a.theta - before), rtol=1e-9, atol=1e-18)
