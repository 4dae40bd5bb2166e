"""Pins for the oracle's GEMMs, epilogue, backward and whole-operator driver (CPU only)."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import qsync_oracle as orc
from tests import bigint_ref as ref

INT8, FP16, FP32 = orc.INT8, orc.FP16, orc.FP32


def _codes(rng, shape):
    return rng.integers(-127, 128, size=shape, dtype=np.int8)


def test_int_gemm_matches_python_integers():
    rng = np.random.default_rng(0)
    for m, n, k in [(1, 1, 1), (3, 5, 7), (8, 8, 8), (4, 2, 33)]:
        a, b = _codes(rng, (m, k)), _codes(rng, (n, k))
        acc, ovf = orc.int_gemm_nt(a, b)
        assert acc.dtype == np.int32 and not ovf
        assert acc.tolist() == ref.gemm_nt(a.tolist(), b.tolist())


def test_int_gemm_medium_against_int64_einsum():
    rng = np.random.default_rng(1)
    a, b = _codes(rng, (70, 1000)), _codes(rng, (45, 1000))
    acc, ovf = orc.int_gemm_nt(a, b)
    want = np.einsum("ik,jk->ij", a.astype(np.int64), b.astype(np.int64))
    np.testing.assert_array_equal(acc.astype(np.int64), want)
    assert not ovf


def test_int32_wraparound_is_reported():
    k = 133145                                   # 127*127*k just exceeds 2^31 - 1
    a = np.full((2, k), 127, np.int8); a[1] = -127
    b = np.full((1, k), 127, np.int8)
    acc, ovf = orc.int_gemm_nt(a, b)
    assert ovf
    assert int(acc[0, 0]) == ref.wrap_i32(127 * 127 * k) and int(acc[0, 0]) < 0
    assert int(acc[1, 0]) == ref.wrap_i32(-127 * 127 * k)
    acc2, ovf2 = orc.int_gemm_nt(a[:, :133144], b[:, :133144])
    assert not ovf2 and int(acc2[0, 0]) == 127 * 127 * 133144


@pytest.mark.parametrize("wgran", ["tensor", "row"])
def test_forward_identity_of_prop2_proof(wgran):
    """q_v q_w sum(v_q w_q) + b == sum(v_hat w_hat) + b with v_hat, w_hat the dequantized tensors."""
    rng = np.random.default_rng(2)
    x = rng.standard_normal((9, 40)).astype(np.float32)
    w = (rng.standard_normal((6, 40)) * rng.uniform(0.01, 0.1, (6, 1))).astype(np.float32)
    bias = rng.standard_normal(6).astype(np.float32)
    sx, ix = orc.scales_from_amax(orc.absmax(x))
    sw, iw = orc.scales_from_amax(orc.absmax(w, wgran))
    xq, wq = orc.quantize_int(x, ix), orc.quantize_int(w, iw, wgran)
    y, acc, _ = orc.qlinear_fwd(INT8, xq, sx, wq, sw, bias, np.float64)
    xh = [[Fraction(int(c)) * Fraction(float(sx[0])) for c in row] for row in xq]
    wh = [[Fraction(int(c)) * Fraction(float(sw[j] if wgran == "row" else sw[0])) for c in row]
          for j, row in enumerate(wq)]
    exact = ref.gemm_nt(xh, wh)
    for i in range(9):
        for j in range(6):
            want = float(exact[i][j] + Fraction(float(bias[j])))
            assert y[i, j] == pytest.approx(want, rel=1e-12, abs=1e-15)
    # fp32 / fp16 outputs are that value rounded once
    y32, _, _ = orc.qlinear_fwd(INT8, xq, sx, wq, sw, bias, np.float32)
    np.testing.assert_array_equal(y32, y.astype(np.float32))
    # and it approximates the unquantized product within the quantization-noise envelope
    full = x.astype(np.float64) @ w.astype(np.float64).T + bias
    swv = sw if wgran == "row" else np.full(6, sw[0])
    bound = 0.5 * (sx[0] * np.abs(w).sum(1) + swv * np.abs(x).sum(1)[:, None]) + 0.25 * 40 * sx[0] * swv
    assert np.all(np.abs(y - full) <= bound * 1.01)


def _fsum_nt(a, b):
    return np.array([[math.fsum(float(p) * float(q) for p, q in zip(ai, bj)) for bj in b] for ai in a])


def test_float_paths_match_textbook_loops():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 19)).astype(np.float32)
    w = rng.standard_normal((4, 19)).astype(np.float32)
    bias = rng.standard_normal(4).astype(np.float32)
    # FP32 tag == naive matmul
    y, acc, ovf = orc.qlinear_fwd(FP32, x, None, w, None, bias, np.float64)
    assert acc is None and not ovf
    np.testing.assert_allclose(y, _fsum_nt(x, w) + bias.astype(np.float64), rtol=1e-14, atol=1e-15)
    y32, _, _ = orc.qlinear_fwd(FP32, x, None, w, None, None, np.float32)
    np.testing.assert_allclose(y32, orc.naive_matmul_nt_f32(x, w), rtol=2e-6, atol=2e-6)
    np.testing.assert_allclose(y32, x @ w.T, rtol=2e-6, atol=2e-6)
    # FP16 tag == exact product of the rounded inputs
    xh, wh = orc.cast_fp16(x), orc.cast_fp16(w)
    yh, _, _ = orc.qlinear_fwd(FP16, xh, None, wh, None, bias, np.float64)
    np.testing.assert_allclose(yh, _fsum_nt(xh, wh) + bias.astype(np.float64), rtol=1e-14, atol=1e-15)
    with pytest.raises(AssertionError):
        orc.qlinear_fwd(FP16, x, None, w, None, None)       # operands must already be cast


def test_backward_contractions_and_layouts():
    """Non-square shapes: a transposed operand or a swapped index cannot pass."""
    rng = np.random.default_rng(4)
    m, n, k = 6, 4, 9
    dyq, xq, wqb = _codes(rng, (m, n)), _codes(rng, (m, k)), _codes(rng, (n, k))
    sdy, sx = np.float32([0.003]), np.float32([0.02])
    swb = rng.uniform(0.001, 0.002, k).astype(np.float32)
    dy = rng.standard_normal((m, n)).astype(np.float32)
    out = orc.qlinear_bwd(INT8, dyq, sdy, xq, sx, wqb, swb, dy, np.float64, np.float64)
    acc_dx = [[sum(int(dyq[i, j]) * int(wqb[j, t]) for j in range(n)) for t in range(k)] for i in range(m)]
    acc_dw = [[sum(int(dyq[i, j]) * int(xq[i, t]) for i in range(m)) for t in range(k)] for j in range(n)]
    assert out["acc_dx"].tolist() == acc_dx and out["acc_dw"].tolist() == acc_dw
    assert out["dx"].shape == (m, k) and out["dw"].shape == (n, k)
    for i in range(m):
        for t in range(k):
            assert out["dx"][i, t] == pytest.approx(acc_dx[i][t] * float(sdy[0]) * float(swb[t]), rel=1e-12)
    for j in range(n):
        for t in range(k):
            assert out["dw"][j, t] == pytest.approx(acc_dw[j][t] * float(sdy[0]) * float(sx[0]), rel=1e-12)
    np.testing.assert_allclose(out["db"], [math.fsum(map(float, dy[:, j])) for j in range(n)], rtol=1e-6)
    # per-tensor backward scale
    out_t = orc.qlinear_bwd(INT8, dyq, sdy, xq, sx, wqb, np.float32([0.5]), None, np.float64, np.float64)
    np.testing.assert_allclose(out_t["dx"], np.array(acc_dx) * float(sdy[0]) * 0.5, rtol=1e-12)
    assert out_t["db"] is None
    # float tags
    dyf = rng.standard_normal((m, n)).astype(np.float32)
    xf = rng.standard_normal((m, k)).astype(np.float32)
    wf = rng.standard_normal((n, k)).astype(np.float32)
    o32 = orc.qlinear_bwd(FP32, dyf, None, xf, None, wf, None, dyf, np.float64, np.float64)
    np.testing.assert_allclose(o32["dx"], _fsum_nt(dyf, wf.T), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(o32["dw"], _fsum_nt(dyf.T, xf.T), rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("tag", [INT8, FP16, FP32])
def test_operator_driver_close_to_float_operator(tag):
    """Whole operator vs the unquantized fp64 operator: within the Prop. 2 noise scale."""
    rng = np.random.default_rng(5)
    m, n, k = 48, 40, 64
    x = rng.standard_normal((m, k)).astype(np.float32)
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    b = rng.standard_normal(n).astype(np.float32) * 0.1
    dy = (rng.standard_normal((m, n)) * 1e-2).astype(np.float32)
    r = orc.operator_fwd_bwd(tag, x, w, b, dy, "row", "stochastic", seed=9, dx_dtype=np.float32)
    y0 = x.astype(np.float64) @ w.T + b
    dx0 = dy.astype(np.float64) @ w
    dw0 = dy.astype(np.float64).T @ x
    tol = {INT8: 0.03, FP16: 2e-3, FP32: 1e-6}[tag]
    for got, want in [(r["y"], y0), (r["dx"], dx0), (r["dw"], dw0)]:
        assert np.abs(got - want).max() <= tol * np.abs(want).max()
    np.testing.assert_allclose(r["db"], dy.sum(0), rtol=1e-5, atol=1e-7)
    assert not r["overflow"]
    if tag == INT8:
        # per-output-channel weights: the backward re-quantizes W with one scale per input feature
        assert r["sw"].shape == (n,) and r["swb"].shape == (k,)
        assert r["wqb"].shape == (n, k) and np.abs(r["wqb"]).max(axis=0).min() == 127


def test_fp16_backward_of_int8_forward_reduces_to_exact_integer_products():
    """Pin for the paper's INT8-forward / FP16-backward pairing.  With power-of-two scales and small codes
    every dequantized operand and every product is exact in binary16/double, so dX and dW must equal the
    integer matrix products scaled by the (exact) scales: a transposed operand, a missing dequantize
    factor or the wrong scale granularity cannot pass."""
    rng = np.random.default_rng(21)
    m, n, k = 7, 5, 11
    xq = rng.integers(-8, 9, (m, k)).astype(np.int8)
    wq = rng.integers(-8, 9, (n, k)).astype(np.int8)
    dy = (rng.integers(-16, 17, (m, n)) / 64.0).astype(np.float32)      # exact in binary16
    sx = np.float32([0.25])
    sw_row = (2.0 ** rng.integers(-4, 1, n)).astype(np.float32)
    for w_gran, sw in (("row", sw_row), ("tensor", np.float32([0.125]))):
        out = orc.fp16_backward_of_int8_forward(xq, sx, wq, sw, w_gran, dy, np.float64, np.float64)
        swn = sw if w_gran == "row" else np.repeat(sw, n)
        W = [[int(wq[j, t]) * float(swn[j]) for t in range(k)] for j in range(n)]
        X = [[int(xq[i, t]) * 0.25 for t in range(k)] for i in range(m)]
        dx = [[math.fsum(float(dy[i, j]) * W[j][t] for j in range(n)) for t in range(k)] for i in range(m)]
        dw = [[math.fsum(float(dy[i, j]) * X[i][t] for i in range(m)) for t in range(k)] for j in range(n)]
        assert out["dx"].tolist() == dx and out["dw"].tolist() == dw
        assert out["xh"].dtype == np.float16 and out["wh"].dtype == np.float16 and out["dyh"].dtype == np.float16
        np.testing.assert_allclose(out["db"], dy.astype(np.float64).sum(0), rtol=1e-6)


def test_fp16_backward_of_int8_forward_error_against_float_operator():
    """On Gaussian data the paper's pairing tracks the unquantized backward within the quantization noise
    of the saved codes (rounding of x and w to 8 bits, then to binary16), and is closer to it than the
    INT8 backward, whose gradient is also quantized."""
    rng = np.random.default_rng(22)
    m, n, k = 64, 48, 80
    x = rng.standard_normal((m, k)).astype(np.float32)
    w = (rng.standard_normal((n, k)) * 0.02).astype(np.float32)
    dy = (rng.standard_normal((m, n)) * 1e-2).astype(np.float32)
    r16 = orc.operator_fwd_bwd(INT8, x, w, None, dy, "row", "stochastic", seed=3, dx_dtype=np.float32, bwd_tag=FP16)
    r8 = orc.operator_fwd_bwd(INT8, x, w, None, dy, "row", "stochastic", seed=3, dx_dtype=np.float32)
    dx0, dw0 = dy.astype(np.float64) @ w, dy.astype(np.float64).T @ x
    e16 = max(np.abs(r16["dx"] - dx0).max() / np.abs(dx0).max(), np.abs(r16["dw"] - dw0).max() / np.abs(dw0).max())
    e8 = max(np.abs(r8["dx"] - dx0).max() / np.abs(dx0).max(), np.abs(r8["dw"] - dw0).max() / np.abs(dw0).max())
    assert e16 < 0.02 and e16 < e8
    assert np.array_equal(r16["y"], r8["y"]) and np.array_equal(r16["xq"], r8["xq"])     # same forward


def test_gelu_and_its_derivative():
    x = np.linspace(-6, 6, 241)
    g = orc.gelu(x)
    assert g[120] == 0 and abs(g[-1] - 6) < 1e-8 and abs(g[0]) < 1e-8
    h = 1e-5
    num = (orc.gelu(x + h) - orc.gelu(x - h)) / (2 * h)
    np.testing.assert_allclose(orc.gelu_grad(x), num, rtol=1e-6, atol=1e-8)


def test_fp32_operator_against_torch_linear_and_its_autograd():
    """An independent library: torch's CPU linear layer in double and the gradients its autograd derives."""
    import torch
    rng = np.random.default_rng(77)
    x = rng.standard_normal((9, 7)).astype(np.float32)
    w = rng.standard_normal((5, 7)).astype(np.float32)
    b = rng.standard_normal(5).astype(np.float32)
    dy = rng.standard_normal((9, 5)).astype(np.float32)
    r = orc.operator_fwd_bwd(orc.FP32, x, w, b, dy, y_dtype=np.float64, dx_dtype=np.float64, dw_dtype=np.float64)
    xt = torch.tensor(x.astype(np.float64), requires_grad=True)
    wt = torch.tensor(w.astype(np.float64), requires_grad=True)
    bt = torch.tensor(b.astype(np.float64), requires_grad=True)
    yt = torch.nn.functional.linear(xt, wt, bt)
    yt.backward(torch.tensor(dy.astype(np.float64)))
    assert np.allclose(r["y"], yt.detach().numpy(), rtol=1e-13, atol=1e-13)
    assert np.allclose(r["dx"], xt.grad.numpy(), rtol=1e-13, atol=1e-13)
    assert np.allclose(r["dw"], wt.grad.numpy(), rtol=1e-13, atol=1e-13)
    assert np.allclose(r["db"], bt.grad.numpy(), rtol=1e-6, atol=1e-6)
