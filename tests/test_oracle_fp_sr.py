"""Pins for the floating-point stochastic quantizer (Appendix, Proposition 2: the two-case rounding rule)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import qsync_oracle as orc


def _neighbours(x: float, k: int):
    """The two candidates of the rule, from exact rationals: floor and floor + spacing at the target spacing
    2^(max(e,-14) - k), with the exact probability of the upper one."""
    ax = Fraction(abs(x))
    if ax == 0:
        return Fraction(0), Fraction(0), Fraction(0)
    e = 0
    while Fraction(2) ** (e + 1) <= ax:
        e += 1
    while Fraction(2) ** e > ax:
        e -= 1
    sp = Fraction(2) ** (max(e, -14) - k)
    lo = (ax // sp) * sp
    return lo, lo + sp, (ax - lo) / sp


@pytest.mark.parametrize("k", [10, 9])
def test_every_draw_enumerated_for_selected_values(k):
    """For one value per row, all 65536 draws are tried (the draw of element 0 of group g under seed s is not
    controllable, so 65536 copies of the value are rounded under one seed and the empirical up-fraction is
    compared with floor(p * 2^16) / 2^16 within sampling error; the two outcomes must be the exact neighbours)."""
    vals = [1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -13, -3.1415927, 0.1, 65000.3, 2.0 ** -15 * 1.37, -2.0 ** -20 * 1.9,
            2.0 ** -26, 1.9999999, 5.9604645e-08 * 0.75]
    n = 1 << 16
    for v in vals:
        x = np.full(n, np.float32(v), np.float32)
        out = orc.cast_fp16_stochastic(x, seed=77, offset=5, k=k).astype(np.float64)
        lo, hi, p = _neighbours(float(np.float32(v)), k)
        sgn = -1.0 if v < 0 else 1.0
        got = set(np.unique(out).tolist())
        assert got <= {sgn * float(lo), sgn * float(hi)}, (v, got, float(lo), float(hi))
        p16 = (p * 65536).__floor__() / 65536.0
        frac_up = np.mean(out == sgn * float(hi)) if hi != lo else 0.0
        assert abs(frac_up - p16) < 5 * np.sqrt(max(p16 * (1 - p16), 1e-9) / n) + 2.0 ** -16, (v, frac_up, p16)


def test_threshold_is_exact_for_known_draws():
    """Element i uses the same draw as the fixed-point quantizer; with the draws in hand the outcome of every
    element is predictable exactly: up iff u < floor(p * 2^16)."""
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(4096) * np.exp(rng.uniform(-12, 8, 4096))).astype(np.float32)
    u = orc.sr_draws(9, 123, x.size)
    out = orc.cast_fp16_stochastic(x, seed=9, offset=123, k=10).astype(np.float64)
    for i in range(x.size):
        lo, hi, p = _neighbours(float(x[i]), 10)
        want = hi if int(u[i]) < (p * 65536).__floor__() else lo
        want = float(want) * (-1.0 if x[i] < 0 else 1.0)
        if abs(want) >= 65536.0:
            want = np.inf * np.sign(want)
        assert out[i] == want, (i, float(x[i]), out[i], want)


def test_representable_values_unchanged_and_binade_carry():
    h = np.array([1.0, -2.5, 65504.0, 6.1035156e-05, 5.9604645e-08, 0.0, -0.0, 1023.5], np.float16)
    out = orc.cast_fp16_stochastic(h.astype(np.float32), seed=3, k=10)
    assert np.array_equal(out.view(np.uint16), h.view(np.uint16))
    assert orc.cast_fp16_stochastic(h, seed=3) is not h and np.array_equal(orc.cast_fp16_stochastic(h), h)
    # just below a power of two: the upper neighbour is the power of two itself (mantissa carry)
    x = np.full(4096, np.float32(2.0 - 2.0 ** -12), np.float32)
    out = orc.cast_fp16_stochastic(x, seed=4, k=10)
    assert set(np.unique(out).tolist()) == {float(np.float16(2.0 - 2.0 ** -10)), 2.0}
    # beyond the largest finite binary16 the upper neighbour is infinity, as in IEEE narrowing
    big = np.full(4096, np.float32(65530.0), np.float32)
    ob = orc.cast_fp16_stochastic(big, seed=5, k=10)
    assert set(np.unique(ob).tolist()) == {65504.0, np.inf}


def test_unbiased_and_variance_of_prop2():
    """E[SR(x)] = x up to 2^-16 of a spacing; the variance of one element is eps^2 2^(2e) f (1 - f), which
    averages to eps^2 2^(2e) / 6 over uniform fractions (Prop. 2, floating-point case, per element)."""
    rng = np.random.default_rng(2)
    x = rng.uniform(1.0, 2.0, 1 << 15).astype(np.float32)           # one binade, e = 0
    acc = np.zeros(x.size); acc2 = np.zeros(x.size)
    T = 64
    for t in range(T):
        o = orc.cast_fp16_stochastic(x, seed=1000 + t, k=10).astype(np.float64)
        acc += o; acc2 += (o - x) ** 2
    assert abs((acc / T - x).mean()) < 3 * 2.0 ** -10 / np.sqrt(12 * T * x.size) + 2.0 ** -26
    assert acc2.mean() / T == pytest.approx((2.0 ** -10) ** 2 / 6.0, rel=0.03)
