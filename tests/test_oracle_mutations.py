"""Meta-test: plausible mistakes planted in the ORACLE (on the CPU) must be caught by its pins.

Each mutation edits one line of the oracle's source text, loads the result as a throw-away module
and re-runs the decimal brute-force traces (all switch combinations) against it.  At least one
combination has to disagree; otherwise the pins would not notice that mistake.
"""
import importlib.util
import os
import sys
import types

import numpy as np
import pytest

from tests import test_oracle_traces as T

SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "novak_oracle.py")

MUTATIONS = {
    "nesterov_sign": ("g = g + h.beta_n * (g - m_prev)", "g = g + h.beta_n * (m_prev - g)"),
    "nesterov_uses_new_m": ("g = g + h.beta_n * (g - m_prev)", "g = g + h.beta_n * (g - (h.beta1 * m_prev + (1.0 - h.beta1) * g))"),
    "eps_inside_root": ("u = m_hat / (np.sqrt(v_hat) + h.eps)", "u = m_hat / np.sqrt(v_hat + h.eps)"),
    "no_v_bias_correction": ("v_hat = v / s.bc2", "v_hat = v"),
    "double_bias_correction": ("theta = theta * s.decay - alpha_eff * u", "theta = theta * s.decay - alpha_eff / s.bc1 * u"),
    "decay_with_rectified_lr": ("decay = 1.0 - h.lr * h.weight_decay if", "decay = 1.0 - h.lr * r_t * h.weight_decay if"),
    "decay_after_update": ("theta = theta * s.decay - alpha_eff * u", "theta = (theta - alpha_eff * u) * s.decay"),
    "threshold_four": ("if rho_t >= 5.0:", "if rho_t >= 4.0:"),
    "rho_missing_denominator": ("rho_t = rho_inf - 2.0 * t * beta2_t / bc2", "rho_t = rho_inf - 2.0 * t * beta2_t"),
    "r_t_no_sqrt": ("r_t = math.sqrt((rho_t - 4.0)", "r_t = ((rho_t - 4.0)"),
    "second_moment_not_squared": ("(1.0 - b2_t) * g * g", "(1.0 - b2_t) * np.abs(g)"),
    "classical_swapped_weights": ("u = h.beta1 * m_hat + (1.0 - h.beta1) * u", "u = (1.0 - h.beta1) * m_hat + h.beta1 * u"),
    "lookahead_k_minus_1": ("slow_new = slow0 + h.la_alpha * delta / h.la_k", "slow_new = slow0 + h.la_alpha * delta / (h.la_k - 1)"),
    "lookahead_sum_of_updates": ("delta += th.astype(np.float64) - slow0", "delta += (th.astype(np.float64) - slow0) / len(st.window)"),
    "sync_one_step_early": ("return h.lookahead != \"none\" and t % h.la_k == 0", "return h.lookahead != \"none\" and (t + 1) % h.la_k == 0"),
    "coupled_decay_sign": ("g = g + h.weight_decay * theta", "g = g - h.weight_decay * theta"),
    "fallback_keeps_denominator": ("denom_on = (h.unrect_fallback == \"adam_denom\")", "denom_on = True"),
    "m_and_v_betas_swapped": ("m = b1_t * m_prev + (1.0 - b1_t) * g", "m = b2_t * m_prev + (1.0 - b2_t) * g"),
}


def _load_mutant(old: str, new: str) -> types.ModuleType:
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation anchor not unique / missing: {old!r}"
    spec = importlib.util.spec_from_loader("novak_oracle_mutant", loader=None)
    mod = importlib.util.module_from_spec(spec)
    sys.modules["novak_oracle_mutant"] = mod      # dataclasses look the module up by name
    try:
        exec(compile(text.replace(old, new), "novak_oracle_mutant", "exec"), mod.__dict__)
    finally:
        sys.modules.pop("novak_oracle_mutant", None)
    return mod


def _n_disagreements(M) -> int:
    bad = 0
    for rectified, decoupled, nesterov, lookahead, fallback in T.COMBOS:
        if not rectified and fallback == "sgdm":
            continue
        h = M.Hyper(lr=float(T.HP["lr"]), beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.01, beta_n=0.8,
                    la_alpha=0.5, la_k=T.K, rectified=rectified, decoupled_decay=decoupled,
                    nesterov=nesterov, lookahead=lookahead, unrect_fallback=fallback)
        want = T._trace(rectified, decoupled, "none" if nesterov == "true" else nesterov, lookahead, fallback)
        try:
            st = M.run([np.array(T.THETA0)], lambda t: [np.array(T.GRADS[t - 1])], T.STEPS, h,
                       state_dtype=np.float64)[0]
        except AssertionError:
            bad += 1
            continue
        for e in range(4):
            th, m, v = want[e]
            ok = (abs(st.theta[e] - th) <= 1e-12 * abs(th) + 1e-18 and abs(st.m[e] - m) <= 1e-12 * abs(m) + 1e-18
                  and abs(st.v[e] - v) <= 1e-12 * abs(v) + 1e-24)
            if not ok:
                bad += 1
                break
    return bad


def test_unmutated_source_passes():
    text = open(SRC).read()
    anchor = "theta = theta * s.decay - alpha_eff * u"
    assert _n_disagreements(_load_mutant(anchor, anchor)) == 0


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name):
    old, new = MUTATIONS[name]
    assert _n_disagreements(_load_mutant(old, new)) > 0, f"pins do not notice mutation {name}"
