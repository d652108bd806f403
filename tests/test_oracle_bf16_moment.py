"""Pins for the oracle's bfloat16 first-moment mode: the rounding itself (against torch's conversion and
hand-made tie cases), a brute force in exact rational arithmetic, and the comparison policy of
tests/harness.py (which roundings may go either way) against an fp32 emulation."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import novak_oracle as O


def test_round_to_bf16_matches_library_conversion_on_fp32_inputs():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 1e-6, 5000), rng.normal(0, 1e6, 5000)]).astype(np.float32)
    want = torch.tensor(x).to(torch.bfloat16).float().numpy()
    got = O.round_to_bf16(x.astype(np.float64))
    assert np.array_equal(got.astype(np.float32), want)


def test_round_to_bf16_ties_to_even_and_single_rounding():
    # 1 + 2^-8 is exactly half way between bf16 neighbours 1 and 1 + 2^-7: ties to even -> 1
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2 * 2.0 ** -7   # tie -> even mantissa
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1.0 + 2.0 ** -7
    # a value that double rounding (via fp32) would get wrong: just below the midpoint by less than an fp32 ulp
    x = 1.0 + 2.0 ** -8 - 2.0 ** -30
    assert np.float32(x) == np.float32(1.0 + 2.0 ** -8)          # fp32 rounds it up onto the midpoint
    assert O.round_to_bf16(np.array([x]))[0] == 1.0              # one rounding from the exact value: down
    assert O.round_to_bf16(np.array([0.0, -0.0])).tolist() == [0.0, 0.0]
    # binade edges: the value just below a power of two rounds up onto it
    assert O.round_to_bf16(np.array([2.0 - 2.0 ** -9, -(4.0 - 2.0 ** -8)])).tolist() == [2.0, -4.0]


def _rne_bf16_fraction(x: Fraction) -> Fraction:
    """Independent bf16 rounding on exact rationals (8 significant bits, ties to even)."""
    if x == 0:
        return x
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = 0
    while a >= 2:
        a /= 2; e += 1
    while a < 1:
        a *= 2; e -= 1
    scaled = a * 128                       # 128 <= scaled < 256
    fl = scaled.numerator // scaled.denominator
    rem = scaled - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return sign * Fraction(fl, 128) * (Fraction(2) ** e)


def test_bf16_moment_trajectory_in_exact_arithmetic():
    """m_t = rne_bf16(beta1 m_{t-1} + (1-beta1) g~_t) with the Nesterov approximation, in rationals."""
    b1, bn = Fraction(9, 10), Fraction(4, 5)
    grads = [Fraction(1, 128), Fraction(-3, 1024), Fraction(5, 512), Fraction(1, 3), Fraction(-7, 9), Fraction(11, 4096), Fraction(2, 7)]
    m = Fraction(0)
    ms = []
    for g in grads:
        gt = g + bn * (g - m)
        m = _rne_bf16_fraction(b1 * m + (1 - b1) * gt)
        ms.append(float(m))
    h = O.Hyper(lr=1e-3, beta1=0.9, beta2=0.999, weight_decay=0.0, beta_n=0.8, rectified=False, nesterov="approx",
                lookahead="none", moment_dtype="bf16_m")
    st = O.init_state(np.zeros(1), h, np.float64)
    for t, g in enumerate(grads, 1):
        O.step(st, np.array([float(g)]), t, h)
        assert st.m[0] == ms[t - 1], t
    # every stored m is a bfloat16 value
    assert float(torch.tensor(st.m[0], dtype=torch.float32).to(torch.bfloat16).float()) == st.m[0]


def test_bf16_moment_changes_only_m_storage():
    rng = np.random.default_rng(5)
    th = rng.normal(0, 0.02, 4096)
    gs = [rng.normal(0, 1e-2, 4096) for _ in range(6)]
    a = O.run([th], lambda t: gs[t - 1], 6, O.Hyper(lookahead="none", moment_dtype="bf16_m"))[0]
    b = O.run([th], lambda t: gs[t - 1], 6, O.Hyper(lookahead="none"))[0]
    rel = np.abs(a.m - b.m) / np.maximum(np.abs(b.m), 1e-12)
    assert 1e-4 < np.median(rel) < 2e-2          # bf16 keeps ~3 significant digits of m
    assert np.max(np.abs(a.theta - b.theta)) < 1e-4 and np.max(np.abs(a.theta - b.theta)) > 0
    # the trace holds the exact m_t of the last step, and the stored one is its rounding
    assert np.array_equal(a.m.astype(np.float64), O.round_to_bf16(a.trace.m_exact))
    assert np.any(a.trace.m_exact != a.m)


def test_stored_m_stands_in_for_the_oracles_own_rounding():
    """stored_m replaces the rounded m_t in Eq. 5 / 17 / 24 of the same step and is what gets stored; the
    exact m_t in the trace does not depend on it, and passing the oracle's own rounding changes nothing."""
    h = O.Hyper(lookahead="none", weight_decay=0.0, moment_dtype="bf16_m", rectified=False, nesterov="none")
    g = np.array([0.3, -0.2, 0.05, 1.0])
    a = O.init_state(np.zeros(4), h, np.float64)
    O.step(a, g, 1, h)
    b = O.init_state(np.zeros(4), h, np.float64)
    O.step(b, g, 1, h, stored_m=a.m)
    assert np.array_equal(a.theta, b.theta) and np.array_equal(a.m, b.m)
    up = a.m + np.ldexp(1.0, np.frexp(a.m)[1] - 8) * np.sign(a.m)          # one bfloat16 ulp further out
    c = O.init_state(np.zeros(4), h, np.float64)
    s = O.step(c, g, 1, h, stored_m=up)
    assert np.array_equal(c.m, up) and np.array_equal(c.trace.m_exact, a.trace.m_exact)
    v_hat = (1 - h.beta2) * g * g / s.bc2
    np.testing.assert_allclose(c.theta, -h.lr * (up / s.bc1) / (np.sqrt(v_hat) + h.eps), rtol=1e-14)
    assert np.array_equal(c.v, a.v)


def test_midpoint_policy_covers_every_disagreement_with_an_fp32_evaluation():
    """The harness's policy is a claim about fp32 arithmetic: Eq. 13 and Eq. 1 evaluated in fp32 (fused
    multiply-adds emulated through double) and rounded to bfloat16 must land inside the policy's range
    at every element; away from midpoints that range is the oracle's own rounding alone; and the
    elements where it is wider must stay rare.  Each step starts from the fp32 evaluation's own stored m
    (a common state)."""
    import workloads as W
    from tests import harness as H
    f32 = np.float32
    n, steps = 1 << 15, 30

    def fma(a, b, c):
        return (a.astype(np.float64) * np.float64(b) + c.astype(np.float64)).astype(f32)

    h = O.Hyper(lookahead="none", weight_decay=1e-2, moment_dtype="bf16_m")
    st = O.init_state(W.host_params([n], 42)[0], h)
    m = np.zeros(n, f32)
    differing, wide = 0, 0
    for t in range(1, steps + 1):
        g = W.host_grads([n], t, 1e-2, 42)[0]
        st.m = m.copy()                                            # common state
        m_prev = m.astype(np.float64)
        gt = fma((g - m).astype(f32), f32(0.9), g)                 # Eq. 13
        m = W.round_to_bf16(fma((gt - m).astype(f32), f32(1.0 - 0.9), m))   # Eq. 1, then the storage rounding
        O.step(st, g, t, h, stored_m=m)
        lo, hi = H.bf16_rounding_range(st.trace, m_prev, h.beta1)
        own = O.round_to_bf16(st.trace.m_exact)
        assert np.all((lo <= m) & (m <= hi)), t
        assert np.all((lo <= own) & (own <= hi)), t
        assert np.all(m[lo == hi] == own[lo == hi]), t             # bit-identical wherever the range is one value
        differing += int((m != own).sum())
        wide += int((lo != hi).sum())
    assert differing > 0                       # the situation the policy exists for does occur
    assert wide / (n * steps) < H.NEAR_MIDPOINT_SHARE["f32"]


def test_rounding_range_is_one_value_away_from_midpoints_and_two_near_them():
    from tests.harness import bf16_rounding_range
    z = np.zeros(3)
    # m_exact = 1 + 2^-8 (a midpoint), 1 + 2^-8 + 2^-20 (2^-20 above it: outside fp32 error), 1.0 (a bfloat16 value)
    tr = O.StepTrace(z, z, z, np.array([1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0]), z, 1.0)
    lo, hi = bf16_rounding_range(tr, z, 0.9)
    assert (lo[0], hi[0]) == (1.0, 1.0 + 2.0 ** -7)
    assert lo[1] == hi[1] == 1.0 + 2.0 ** -7
    assert lo[2] == hi[2] == 1.0
