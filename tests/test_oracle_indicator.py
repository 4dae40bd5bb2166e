"""Pins for the indicator statistics and the variance-increment formula (Indicator section, Prop. 2 / Prop. 3)."""
import math

import numpy as np
import pytest

from oracle import qsync_oracle as orc


def test_tensor_stats_against_exact_sums():
    rng = np.random.default_rng(0)
    for dtype in (np.float32, np.float16):
        x = (rng.standard_normal((37, 53)) * 3).astype(dtype)
        st = orc.tensor_stats(x)
        assert st["sumsq"] == pytest.approx(math.fsum(float(v) * float(v) for v in x.reshape(-1)), rel=1e-14)
        assert st["amax"] == max(abs(float(v)) for v in x.reshape(-1))
        assert st["D"] == 37 * 53
        assert 2.0 ** st["e"] <= st["amax"] < 2.0 ** (st["e"] + 1)
    z = orc.tensor_stats(np.zeros((4, 4), np.float32))
    assert z["sumsq"] == 0 and z["amax"] == 0 and z["e"] == -126
    assert orc.effective_exponent(1.0) == 0 and orc.effective_exponent(0.99) == -1 and orc.effective_exponent(6.5) == 2


def test_variance_increment_hand_computed_cases():
    """Small integers so that every term can be checked by hand; swapping two tensors, dropping a factor
    or mixing up the fixed- and floating-point branches changes the numbers."""
    x = dict(sumsq=2.0, amax=1.0, e=0, D=3)        # parameter
    v = dict(sumsq=5.0, amax=2.5, e=1, D=7)        # activation
    g = dict(sumsq=11.0, amax=0.3, e=-2, D=7)      # activation gradient
    r = orc.variance_increment("fixed", x, v, g, q_x=0.5, q_v=0.25, eps=2.0 ** -3, gamma=2.0, d_o=3, d_L=10)
    s_fp = (2.0 * 0.0625 * 7 + 5.0 * 0.25 * 3) / 6
    s_bp = (11.0 * 0.0625 * 7 + 5.0 * (2.0 ** -4) * (2.0 ** -6) * 7) / 6
    assert r["sigma_fp"] == pytest.approx(s_fp, rel=1e-15) and r["sigma_bp"] == pytest.approx(s_bp, rel=1e-15)
    assert r["omega"] == pytest.approx(4.0 * 3 * s_fp + 7 * s_bp, rel=1e-15)
    r = orc.variance_increment("float", x, v, g, eps=2.0 ** -3, gamma=1.0, d_o=2, d_L=5)
    s_fp = (2.0 ** -6) * (2.0 * 4.0 * 7 + 5.0 * 1.0 * 3) / 6
    s_bp = (2.0 ** -6) * (11.0 * 4.0 * 7 + 5.0 * (2.0 ** -4) * 7) / 6
    assert r["sigma_fp"] == pytest.approx(s_fp, rel=1e-15) and r["sigma_bp"] == pytest.approx(s_bp, rel=1e-15)
    assert r["omega"] == pytest.approx(2 * s_fp + 3 * s_bp, rel=1e-15)
    with pytest.raises(ValueError):
        orc.variance_increment("other", x, v, g)


def test_fixed_point_forward_term_matches_measured_quantization_variance():
    """sigma_fp is the first-order variance of the operator output under stochastic rounding of both
    operands (Prop. 2: q^2/6 per element).  Summed over the outputs of a linear operator whose weight rows all
    have the same squared norm, the measured variance of Y = X W^T under SR of X and of W equals
    (|W_row|^2 q_v^2 D_v + |v|^2 q_x^2 D_x) / 6 with x one weight row: checked by simulation."""
    rng = np.random.default_rng(3)
    m, k = 16, 64
    v = rng.uniform(-1, 1, (m, k)).astype(np.float32)
    w = rng.uniform(-1, 1, (1, k)).astype(np.float32)                     # one output feature
    q_v, q_x = 2.0 ** -5, 2.0 ** -6
    inv_v, inv_x = np.float32([1 / q_v]), np.float32([1 / q_x])
    ys = []
    for seed in range(400):
        vq = orc.quantize_int(v, inv_v, "tensor", "stochastic", seed=seed, offset=0).astype(np.float64) * q_v
        wq = orc.quantize_int(w, inv_x, "tensor", "stochastic", seed=10_000 + seed, offset=0).astype(np.float64) * q_x
        ys.append(vq @ wq.T)
    var_total = np.var(np.stack(ys), axis=0, ddof=1).sum()               # summed over the m outputs
    x_st, v_st = orc.tensor_stats(w), orc.tensor_stats(v)
    # per element variance q^2/6: sum_i x_i^2 * q_v^2/6 for each of the m rows + sum_{r,i} v_ri^2 * q_x^2/6
    predicted = (x_st["sumsq"] * q_v ** 2 * m + v_st["sumsq"] * q_x ** 2) / 6.0
    assert var_total == pytest.approx(predicted, rel=0.15)
    # the indicator's expression carries the dimensionalities D as weights; with D_v -> m and D_x -> 1 it is this sum
    r = orc.variance_increment("fixed", x_st | {"D": 1}, v_st | {"D": m}, v_st, q_x=q_x, q_v=q_v)
    assert r["sigma_fp"] == pytest.approx(predicted, rel=1e-12)
