"""Decimal brute force of the full-features step (every optional phase at once) and a mutation
meta-test over the oracle's research-mode code.

The brute force is written from the equations with Python's `decimal` (50 digits), scalar by scalar,
and shares nothing with the oracle: clipping on the global norm (section 7.3), centralization (Eq. 26),
coupled decay, the Nesterov approximation (Eq. 13), scheduled betas in the moment updates (Eq. 3-4),
bias correction and rectification with the base betas (Eq. 5-9), the trust ratio on the unmasked
direction (Eq. 19, 25), the automatic rate from the norms of the gradient as handed in (Eq. 20-23), the
sparse mask (Eq. 27) before the classical blend (Eq. 16), the update (Eq. 24, 24a) and the averaging
lookahead sync (Eq. 30-31).
"""
from decimal import Decimal as D, getcontext

import numpy as np
import pytest

from oracle import novak_oracle as O
from tests.test_oracle_mutations import _load_mutant

getcontext().prec = 50

# tensor 0 is a 2 x 3 matrix (centralized per row when the switch is on), tensor 1 a vector
# tensor 2's norm ratio sits above the trust ratio's upper clip, tensor 3's below the lower one
THETA0 = [[0.25, -0.015625, 0.001953125, -3.0, 0.5, 0.125], [1.5, -0.75, 0.03125], [64.0, -32.0], [0.0009765625, -0.001953125]]
ROWS = [2, 0, 0, 0]
GRADS = [
    [[0.0078125, -0.001953125, 0.03125, 0.5, -0.25, 0.0625], [0.25, -0.125, 0.0625], [0.125, -0.0625], [0.03125, 0.25]],
    [[-0.00390625, -0.0009765625, 0.000244140625, 0.25, 0.125, -0.5], [-0.5, 0.03125, 0.015625], [-0.25, 0.03125], [0.125, -0.0625]],
    [[0.005859375, 0.001953125, -0.000244140625, -0.75, 0.0625, 0.03125], [0.125, 0.25, -0.0078125], [0.0625, 0.125], [-0.25, 0.5]],
    [[0.0009765625, -0.0029296875, 0.0001220703125, 0.125, -0.015625, 0.25], [0.0625, -0.375, 0.5], [0.5, -0.25], [0.0625, 0.03125]],
    [[-0.0068359375, 0.00048828125, 0.015625, 0.375, 0.25, -0.125], [-0.03125, 0.125, 0.25], [-0.125, 0.0625], [0.5, -0.125]],
    [[0.0029296875, -0.00146484375, -0.0003662109375, -0.0625, 0.5, 0.0078125], [0.75, 0.5, -0.125], [0.25, 0.5], [-0.03125, 0.0625]],
    [[0.001953125, 0.00244140625, 0.00006103515625, 0.4375, -0.375, 0.0625], [0.25, -0.0625, 0.375], [0.03125, -0.5], [0.25, 0.125]],
]
K, STEPS = 3, 7

CONFIGS = [
    # clip, gc, decoupled, nesterov, adaptive, layer, auto, sparse
    # clip thresholds 0.85 / 0.8 lie inside the range of the gradient norms (0.69 .. 1.18): some steps clip, some do not.
    # ||g|| / ||theta|| is about 0.012: auto_lo = 0.001 leaves Eq. 22 unclipped, the default 0.1 clips it.
    dict(clip=0.85, gc=True, decoupled=True, nesterov="approx", adaptive=True, layer=True, auto=True, sparse=0.45, auto_lo=0.001),
    dict(clip=0.8, gc=True, decoupled=False, nesterov="classical", adaptive=True, layer=True, auto=False, sparse=0.45, auto_lo=0.1),
    dict(clip=0.0, gc=True, decoupled=True, nesterov="none", adaptive=False, layer=False, auto=True, sparse=0.0, auto_lo=0.001),
    dict(clip=0.3, gc=False, decoupled=True, nesterov="classical", adaptive=False, layer=True, auto=True, sparse=0.7, auto_lo=0.1),
    dict(clip=0.0, gc=False, decoupled=False, nesterov="approx", adaptive=True, layer=False, auto=False, sparse=0.45, auto_lo=0.1),
]
TAU1, TAU2 = D(4), D(9)


def _brute(cfg):
    lr, b1, b2, eps, wd, bn, la, gam = D("0.001"), D("0.9"), D("0.99"), D("1e-8"), D("0.01"), D("0.8"), D("0.5"), D("0.1")
    th = [[D(x) for x in t] for t in THETA0]
    m = [[D(0)] * len(t) for t in THETA0]
    v = [[D(0)] * len(t) for t in THETA0]
    slow0 = [list(t) for t in th]
    window = [[] for _ in th]
    gbar = tbar = D(0)
    closest = D(1)        # how close any |u| came to the sparse threshold (relative)
    for t in range(1, STEPS + 1):
        bc1, bc2 = 1 - b1 ** t, 1 - b2 ** t
        rho_inf = 2 / (1 - b2) - 1
        rho_t = rho_inf - 2 * t * b2 ** t / bc2
        r = ((rho_t - 4) * (rho_t - 2) * rho_inf / ((rho_inf - 4) * (rho_inf - 2) * rho_t)).sqrt() if rho_t >= 5 else D(1)
        b1t = b1 * (1 - (-D(t) / TAU1).exp()) if cfg["adaptive"] else b1
        b2t = b2 * (1 - (-D(t) / TAU2).exp()) if cfg["adaptive"] else b2
        raw = [[D(x) for x in tens] for tens in GRADS[t - 1]]
        gnorm = sum(x * x for tens in raw for x in tens).sqrt()
        a_auto = D(1)
        if cfg["auto"]:
            tn = sum(x * x for tens in th for x in tens).sqrt()
            gbar = gam * gnorm + (1 - gam) * gbar
            tbar = gam * tn + (1 - gam) * tbar
            a_auto = min(max(gbar / tbar, D(str(cfg["auto_lo"]))), D(2))
        c = D(str(cfg["clip"]))
        gscale = c / gnorm if (c > 0 and gnorm > c) else D(1)
        for i in range(len(th)):
            n = len(th[i])
            g = [x * gscale for x in raw[i]]
            if cfg["gc"] and ROWS[i] >= 1:
                cols = n // ROWS[i]
                for rr in range(ROWS[i]):
                    mean = sum(g[rr * cols:(rr + 1) * cols]) / cols
                    for e in range(rr * cols, (rr + 1) * cols):
                        g[e] -= mean
            us, mh = [], []
            for e in range(n):
                ge = g[e]
                if not cfg["decoupled"]:
                    ge = ge + wd * th[i][e]
                if cfg["nesterov"] == "approx":
                    ge = ge + bn * (ge - m[i][e])
                m[i][e] = b1t * m[i][e] + (1 - b1t) * ge
                v[i][e] = b2t * v[i][e] + (1 - b2t) * ge * ge
                mh.append(m[i][e] / bc1)
                us.append(mh[e] / ((v[i][e] / bc2).sqrt() + eps))
            trust = D(1)
            if cfg["layer"]:
                nt = sum(x * x for x in th[i]).sqrt()
                nu = sum(x * x for x in us).sqrt()
                eta = nt / nu if (nt > 0 and nu > 0) else D(1)
                trust = min(max(eta, D("0.1")), D(10))
            tau = D(str(cfg["sparse"]))
            for e in range(n):
                u = us[e]
                if tau > 0:
                    closest = min(closest, abs(abs(u) - tau) / tau)
                    if not abs(u) > tau:
                        u = D(0)
                if cfg["nesterov"] == "classical":
                    u = b1 * mh[e] + (1 - b1) * u
                decay = (1 - lr * wd) if cfg["decoupled"] else D(1)
                th[i][e] = th[i][e] * decay - lr * r * trust * a_auto * u
            window[i].append(list(th[i]))
            if t % K == 0:
                for e in range(n):
                    th[i][e] = slow0[i][e] + la * sum(w[e] - slow0[i][e] for w in window[i]) / K
                slow0[i], window[i] = list(th[i]), []
    assert closest > D("1e-6"), "test inputs put a direction on the sparse threshold; pick others"
    return ([[float(x) for x in t] for t in th], [[float(x) for x in t] for t in m], [[float(x) for x in t] for t in v])


def _hyper(M, cfg):
    return M.Hyper(lr=1e-3, beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.01, beta_n=0.8, la_alpha=0.5, la_k=K,
                   rectified=True, decoupled_decay=cfg["decoupled"], nesterov=cfg["nesterov"], lookahead="memory_efficient",
                   layer_adaptation=cfg["layer"], auto_lr=cfg["auto"], clip_threshold=cfg["clip"],
                   sparse_threshold=cfg["sparse"], use_gc=cfg["gc"], adaptive_beta=cfg["adaptive"],
                   beta_tau1=float(TAU1), beta_tau2=float(TAU2), auto_clip=(cfg["auto_lo"], 2.0))


def _agrees(M, cfg, want) -> bool:
    try:
        sts = M.run([np.array(t) for t in THETA0], lambda t: [np.array(g) for g in GRADS[t - 1]], STEPS, _hyper(M, cfg),
                    state_dtype=np.float64, rows=ROWS)
    except (AssertionError, ZeroDivisionError, FloatingPointError, ValueError):
        return False
    for st, th, m, v in zip(sts, *want):
        if not (np.allclose(st.theta, th, rtol=1e-11, atol=1e-18) and np.allclose(st.m, m, rtol=1e-11, atol=1e-20)
                and np.allclose(st.v, v, rtol=1e-11, atol=1e-24)):
            return False
    return True


WANT = None


def _want():
    global WANT
    if WANT is None:
        WANT = [_brute(c) for c in CONFIGS]
    return WANT


@pytest.mark.parametrize("i", range(len(CONFIGS)))
def test_everything_on_matches_decimal_brute_force(i):
    assert _agrees(O, CONFIGS[i], _want()[i])


def test_the_switches_matter():
    """Each optional phase changes the result on these inputs (so agreeing with the brute force is not vacuous)."""
    base = CONFIGS[0]
    full = _brute(base)[0]
    for key, off in (("clip", 0.0), ("gc", False), ("adaptive", False), ("layer", False), ("auto", False), ("sparse", 0.0)):
        other = _brute(dict(base, **{key: off}))[0]
        # (the direction is nearly invariant to a rescaled gradient, so clipping moves theta least)
        assert max(abs(a - b) for x, y in zip(full, other) for a, b in zip(x, y)) > (1e-8 if key == "clip" else 1e-7), key


MUTATIONS = {
    "trust_ratio_inverted": ("eta = n_theta / n_u if", "eta = n_u / n_theta if"),
    "trust_ratio_unclipped": ("return min(max(eta, h.trust_clip[0]), h.trust_clip[1])", "return eta"),
    "trust_ratio_of_squares": ("n_u = math.sqrt(float(np.dot(u, u)))", "n_u = float(np.dot(u, u))"),
    "trust_ratio_after_mask": (
        "    lam_trust = trust_ratio(theta, u, h) if h.layer_adaptation else 1.0   # Eq. 19 / 25 (Phase 7)\n",
        "    lam_trust = trust_ratio(theta, np.where(np.abs(u) > h.sparse_threshold, u, 0.0), h) if h.layer_adaptation else 1.0\n"),
    "auto_lr_inverted": ("aux.g_bar / aux.theta_bar, h.auto_clip[0]", "aux.theta_bar / aux.g_bar, h.auto_clip[0]"),
    "auto_lr_ema_weights_swapped": ("aux.g_bar = gam * math.sqrt(g2) + (1.0 - gam) * aux.g_bar", "aux.g_bar = (1.0 - gam) * math.sqrt(g2) + gam * aux.g_bar"),
    "auto_lr_squared_norm": ("aux.theta_bar = gam * math.sqrt(t2)", "aux.theta_bar = gam * t2"),
    "auto_lr_dropped": ("alpha_eff = s.step_size * lam_trust * alpha_auto", "alpha_eff = s.step_size * lam_trust"),
    "auto_lr_sees_clipped_gradient": ("        alpha_auto = auto_lr_scale(aux, [st.theta for st in states], grads, h)\n",
                                      "        alpha_auto = auto_lr_scale(aux, [st.theta for st in states], [np.asarray(g) * clip_scale(grads, h) for g in grads], h)\n"),
    "decay_scaled_by_trust": ("theta = theta * s.decay - alpha_eff * u", "theta = theta * (1.0 - (1.0 - s.decay) * lam_trust) - alpha_eff * u"),
    "clip_always_normalises": ("return h.clip_threshold / norm if norm > h.clip_threshold else 1.0", "return h.clip_threshold / norm"),
    "clip_per_tensor": ("        step(st, g, t, h, alpha_auto, g_scale, None if stored_m is None else stored_m[i])",
                        "        step(st, g, t, h, alpha_auto, clip_scale([g], h), None if stored_m is None else stored_m[i])"),
    "centralize_over_rows": ("g2d.mean(axis=1, keepdims=True)", "g2d.mean(axis=0, keepdims=True)"),
    "centralize_whole_tensor": ("g2d.mean(axis=1, keepdims=True)", "g2d.mean()"),
    "centralize_after_nesterov": ("    if h.use_gc and st.rows >= 1:\n", "    if False:\n"),
    "mask_keeps_small": ("u = np.where(np.abs(u) > h.sparse_threshold, u, 0.0)", "u = np.where(np.abs(u) < h.sparse_threshold, u, 0.0)"),
    "mask_on_signed_value": ("u = np.where(np.abs(u) > h.sparse_threshold, u, 0.0)", "u = np.where(u > h.sparse_threshold, u, 0.0)"),
    "schedule_decays_instead_of_warming": ("h.beta1 * (1.0 - math.exp(-t / h.beta_tau1))", "h.beta1 * math.exp(-t / h.beta_tau1)"),
    "schedule_time_scales_swapped": ("h.beta2 * (1.0 - math.exp(-t / h.beta_tau2))", "h.beta2 * (1.0 - math.exp(-t / h.beta_tau1))"),
    "bias_correction_follows_schedule": ("m_hat = m / s.bc1", "m_hat = m / (1.0 - b1_t ** t)"),
}


def test_unmutated_oracle_agrees_everywhere():
    anchor = "alpha_eff = s.step_size * lam_trust * alpha_auto"
    M = _load_mutant(anchor, anchor)
    assert all(_agrees(M, c, w) for c, w in zip(CONFIGS, _want()))


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_in_research_code_is_caught(name):
    old, new = MUTATIONS[name]
    M = _load_mutant(old, new)
    assert not all(_agrees(M, c, w) for c, w in zip(CONFIGS, _want())), f"the brute force does not notice mutation {name}"
