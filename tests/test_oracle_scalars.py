"""Pins for the oracle's per-step scalars (section 4.3, Eq. 6-9; section 4.2, Eq. 5; Prop. 6.4).

None of these re-evaluates Eq. 7 or Eq. 9 in the same floating-point form.  They use what the
mathematics fixes: rho_t is the length of the simple moving average whose centre of mass equals that
of the exponential moving average after t steps (the RAdam construction the paper follows), checked
by brute-force summation; r_t^2 is a ratio of the variance proxy rho/((rho-2)(rho-4)); exact
rational arithmetic for the whole schedule; limits and monotonicity.
"""
from fractions import Fraction

import mpmath
import pytest

from oracle import novak_oracle as O


def _ema_centre_of_mass(beta: Fraction, t: int) -> Fraction:
    """Mean age (1 = newest) of the EMA weights (1-beta)*beta^(t-i), normalised by 1-beta^t."""
    num = sum((1 - beta) * beta ** (t - i) * (t + 1 - i) for i in range(1, t + 1))
    return num / (1 - beta ** t)


@pytest.mark.parametrize("beta2", [Fraction(999, 1000), Fraction(99, 100), Fraction(95, 100)])
def test_rho_t_is_sma_length_with_equal_centre_of_mass(beta2):
    # an SMA of length f has centre of mass (f+1)/2  =>  f = 2*c - 1
    h = O.Hyper(beta2=float(beta2))
    for t in [1, 2, 3, 5, 6, 10, 37, 100, 400]:
        f_exact = 2 * _ema_centre_of_mass(beta2, t) - 1
        s = O.step_scalars(h, t)
        assert s.rho_t == pytest.approx(float(f_exact), rel=1e-11, abs=1e-11)


def test_rho_1_is_one_and_rho_inf_limit():
    for b2 in (0.5, 0.9, 0.99, 0.999, 0.9999):
        h = O.Hyper(beta2=b2)
        assert O.step_scalars(h, 1).rho_t == pytest.approx(1.0, abs=1e-9)
        assert O.step_scalars(h, 1).rho_inf == pytest.approx(2.0 / (1.0 - b2) - 1.0, rel=1e-15)
        # rho_t -> rho_inf, r_t -> 1 (the paper: "as rho_t -> rho_inf, r_t -> 1")
        s = O.step_scalars(h, 10_000_000)
        assert s.rho_t == pytest.approx(s.rho_inf, rel=1e-9)
        assert s.r_t == pytest.approx(1.0, abs=1e-9)


def test_rho_inf_1999_for_default_beta2():
    assert O.step_scalars(O.Hyper(beta2=0.999), 1).rho_inf == pytest.approx(1999.0, rel=1e-12)


@pytest.mark.parametrize("beta2", [0.999, 0.99, 0.95])
def test_first_rectified_step_is_six(beta2):
    """rho_t crosses 5 between t = 5 and t = 6 for the usual beta2 values (rho_t ~ t for small t)."""
    h = O.Hyper(beta2=beta2, rectified=True)
    flags = [O.step_scalars(h, t).rectified_now for t in range(1, 12)]
    assert flags == [False] * 5 + [True] * 6
    for t in range(1, 6):
        s = O.step_scalars(h, t)
        assert s.r_t == 1.0 and s.step_size == h.lr
    # rho_t < t for all t (the EMA has seen only t samples)
    for t in range(2, 50):
        assert O.step_scalars(h, t).rho_t < t


def test_monotone_rho_and_r_bounds_prop_6_4():
    h = O.Hyper(beta2=0.999)
    prev_rho, prev_r = -1.0, 0.0
    for t in range(1, 3000):
        s = O.step_scalars(h, t)
        assert s.rho_t > prev_rho
        prev_rho = s.rho_t
        assert 0.0 < s.r_t <= 1.0
        if s.rectified_now:
            assert s.r_t > prev_r          # r_t increases once rectification is active
            prev_r = s.r_t
        # Prop. 6.4: alpha_eff = step_size / bc1 is bounded by alpha/(1-beta1) above
        assert s.step_size / s.bc1 <= h.lr / (1 - h.beta1) + 1e-18


def test_r_t_squared_is_variance_ratio_in_exact_arithmetic():
    """r_t^2 = C(rho_inf)/C(rho_t), C(rho) = rho/((rho-2)(rho-4)), evaluated in rationals."""
    b2 = Fraction(999, 1000)
    h = O.Hyper(beta2=float(b2))
    rho_inf = 2 / (1 - b2) - 1

    def c(rho):
        return rho / ((rho - 2) * (rho - 4))

    total = mpmath.mpf(0)
    mpmath.mp.dps = 40
    for t in range(1, 101):
        rho_t = 2 * _ema_centre_of_mass(b2, t) - 1
        s = O.step_scalars(h, t)
        if rho_t >= 5:
            r2 = c(rho_inf) / c(rho_t)
            r = mpmath.sqrt(mpmath.mpf(r2.numerator) / mpmath.mpf(r2.denominator))
            assert s.r_t == pytest.approx(float(r), rel=1e-11)
            total += r
        else:
            assert s.r_t == 1.0
            total += 1
    # the sum of r_t over the first 100 steps fixes the constant-gradient trajectory length
    got = sum(O.step_scalars(h, t).r_t for t in range(1, 101))
    assert got == pytest.approx(float(total), rel=1e-11)
    assert 18.0 < got < 19.5   # five unit steps, then r_6 ~ 0.026 rising to r_100 ~ 0.215


def test_bias_correction_log_form_matches_exact_power():
    """1 - beta^t through exp/log (section 5.8) against exact rational powers, small and large t."""
    for beta, fb in ((0.9, Fraction(9, 10)), (0.999, Fraction(999, 1000))):
        for t in (1, 2, 7, 100, 1000, 5000):
            exact = 1 - fb ** t
            exact_f = float(mpmath.mpf(exact.numerator) / mpmath.mpf(exact.denominator))
            assert O.one_minus_pow(beta, t) == pytest.approx(exact_f, rel=2e-13)
    assert O.one_minus_pow(0.0, 3) == 1.0


def test_decay_and_step_size_scalars():
    h = O.Hyper(lr=2e-3, weight_decay=0.05, rectified=False)
    s = O.step_scalars(h, 17)
    assert s.decay == 1.0 - 2e-3 * 0.05 and s.step_size == 2e-3 and s.denom_on
    h2 = O.Hyper(lr=2e-3, weight_decay=0.05, decoupled_decay=False)
    assert O.step_scalars(h2, 17).decay == 1.0
    # fallback reading only matters while rho_t < 5
    assert not O.step_scalars(O.Hyper(unrect_fallback="sgdm"), 3).denom_on
    assert O.step_scalars(O.Hyper(unrect_fallback="sgdm"), 6).denom_on
    assert O.step_scalars(O.Hyper(unrect_fallback="adam_denom"), 3).denom_on


def _decimal_schedule(beta2: str, t: int):
    """Eq. 6, 7, 9 in 50-digit decimal arithmetic (independent of the oracle's floating-point form)."""
    from decimal import Decimal as D, getcontext
    getcontext().prec = 50
    b2 = D(beta2)
    rho_inf = 2 / (1 - b2) - 1
    bt = b2 ** t
    rho_t = rho_inf - 2 * t * bt / (1 - bt)
    r_t = ((rho_t - 4) * (rho_t - 2) * rho_inf / ((rho_inf - 4) * (rho_inf - 2) * rho_t)).sqrt() if rho_t >= 5 else D(1)
    return float(rho_inf), float(rho_t), float(r_t)


def test_schedule_landmarks_of_the_default_configuration():
    """Numbers a reader can check by hand from Eq. 6-9 with beta2 = 0.999: rho_inf = 1999, rho_1..6 =
    1, 1.9995, 2.9987, 3.9975, 4.9960, 5.9942, so the first rectified step is t = 6 (also for 0.99 and
    0.95), r_6 = 0.025821, r_100 = 0.215335, r_10000 = 0.999773, and the r_t of the first 100 steps (1 while
    unrectified) add up to 18.731269 - the factor of the constant-gradient closed form."""
    assert _decimal_schedule("0.999", 1)[0] == pytest.approx(1999.0, rel=1e-14)
    for t, want in zip(range(1, 7), (1.0, 1.9995, 2.9987, 3.9975, 4.9960, 5.9942)):
        assert _decimal_schedule("0.999", t)[1] == pytest.approx(want, abs=6e-5)
    landmarks = {("0.999", 6): 0.025821, ("0.999", 10): 0.048998, ("0.999", 100): 0.215335, ("0.999", 1000): 0.645326,
                 ("0.999", 10000): 0.999773, ("0.99", 6): 0.081679, ("0.99", 100): 0.634117}
    for (b2, t), want in landmarks.items():
        exact = _decimal_schedule(b2, t)
        assert exact[2] == pytest.approx(want, abs=6e-7)
        s = O.step_scalars(O.Hyper(beta2=float(b2)), t)
        assert s.rectified_now and s.r_t == pytest.approx(exact[2], rel=1e-12) and s.rho_t == pytest.approx(exact[1], rel=1e-12)
    for b2 in ("0.999", "0.99", "0.95"):
        h = O.Hyper(beta2=float(b2))
        first = [t for t in range(1, 30) if O.step_scalars(h, t).rectified_now][0]
        assert first == 6 and _decimal_schedule(b2, 5)[1] < 5.0 <= _decimal_schedule(b2, 6)[1]
    total = sum(O.step_scalars(O.Hyper(), t).r_t for t in range(1, 101))
    assert total == pytest.approx(sum(_decimal_schedule("0.999", t)[2] for t in range(1, 101)), rel=1e-12)
    assert total == pytest.approx(18.731269, abs=1e-6)
