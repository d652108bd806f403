"""Pins for the oracle's bfloat16 first-moment mode: the rounding itself (against torch's conversion and
hand-made tie cases) and a brute force in exact rational arithmetic."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import novak_oracle as O


def test_round_to_bf16_matches_library_conversion_on_fp32_inputs():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 1e-6, 5000), rng.normal(0, 1e6, 5000)]).astype(np.float32)
    want = torch.tensor(x).to(torch.bfloat16).float().numpy()
    got, dist = O.round_to_bf16(x.astype(np.float64))
    assert np.array_equal(got.astype(np.float32), want)
    assert np.all((dist >= 0) & (dist <= 0.5))


def test_round_to_bf16_ties_to_even_and_single_rounding():
    # 1 + 2^-8 is exactly half way between bf16 neighbours 1 and 1 + 2^-7: ties to even -> 1
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8]))[0][0] == 1.0
    assert O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0][0] == 1.0 + 2 * 2.0 ** -7   # tie -> even mantissa
    assert O.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40]))[0][0] == 1.0 + 2.0 ** -7
    # a value that double rounding (via fp32) would get wrong: just below the midpoint by less than an fp32 ulp
    x = 1.0 + 2.0 ** -8 - 2.0 ** -30
    assert np.float32(x) == np.float32(1.0 + 2.0 ** -8)          # fp32 rounds it up onto the midpoint
    assert O.round_to_bf16(np.array([x]))[0][0] == 1.0           # one rounding from the exact value: down
    assert O.round_to_bf16(np.array([0.0, -0.0]))[0].tolist() == [0.0, 0.0]
    d = O.round_to_bf16(np.array([1.0 + 2.0 ** -8, 1.0, 1.0 + 2.0 ** -9]))[1]
    assert d.tolist() == [0.0, 0.5, 0.25]


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


def test_bf16_moment_changes_only_m_storage_and_flags_near_midpoints():
    rng = np.random.default_rng(5)
    th = rng.normal(0, 0.02, 4096)
    gs = [rng.normal(0, 1e-2, 4096) for _ in range(6)]
    a = O.run([th], lambda t: gs[t - 1], 6, O.Hyper(lookahead="none", moment_dtype="bf16_m"))[0]
    b = O.run([th], lambda t: gs[t - 1], 6, O.Hyper(lookahead="none"))[0]
    rel = np.abs(a.m - b.m) / np.maximum(np.abs(b.m), 1e-12)
    assert 1e-4 < np.median(rel) < 2e-2          # bf16 keeps ~3 significant digits of m
    assert np.max(np.abs(a.theta - b.theta)) < 1e-4 and np.max(np.abs(a.theta - b.theta)) > 0
    assert a.ambiguous is not None and a.ambiguous.mean() < 0.02
    assert b.ambiguous is None


def test_flags_cover_every_disagreement_with_an_fp32_evaluation():
    """The oracle's flag is a claim about fp32 arithmetic: wherever Eq. 13 and Eq. 1 evaluated in fp32
    (fused multiply-adds emulated through double) round to another bfloat16 than the exact value, the
    element must have been flagged; and the flags must stay rare."""
    import workloads as W
    f32 = np.float32
    n, steps = 1 << 15, 30

    def fma(a, b, c):
        return (a.astype(np.float64) * np.float64(b) + c.astype(np.float64)).astype(f32)

    h = O.Hyper(lookahead="none", weight_decay=1e-2, moment_dtype="bf16_m")
    st = O.init_state(W.host_params([n], 42)[0], h)
    m = np.zeros(n, f32)
    differing = 0
    for t in range(1, steps + 1):
        g = W.host_grads([n], t, 1e-2, 42)[0]
        O.step(st, g, t, h)
        gt = fma((g - m).astype(f32), f32(0.9), g)                 # Eq. 13
        m = W.round_to_bf16(fma((gt - m).astype(f32), f32(1.0 - 0.9), m))   # Eq. 1, then the storage rounding
        diff = m != st.m
        differing = max(differing, int(diff.sum()))
        assert not np.any(diff & ~st.ambiguous), t
    assert differing > 0                       # the situation the flags exist for does occur
    assert st.ambiguous.mean() < 1.5 * steps * 8e-4
