"""Pins for the oracle's 3x3 convolution (forward, data gradient, weight gradient): CPU only.

Independent checks: scipy's 2-D correlation per channel pair, six-deep brute-force loops over the
definition, single-tap kernels (pure shifts with zero fill), a hand-worked example, the adjoint
identities <conv(X,W), dY> = <X, dgrad(dY,W)> = <W, wgrad(dY,X)> (exact in integers), the lowering
to a GEMM over the patch matrix (the definition of the conv-as-GEMM workload), and finite differences.
"""
import numpy as np
import pytest
from scipy import signal

from oracle import qsync_oracle as orc
from paper_2407_02327_amd import workloads as wl


def codes(rng, shape):
    return rng.integers(-127, 128, shape).astype(np.int8)


def test_forward_matches_scipy_correlation_per_channel_pair():
    rng = np.random.default_rng(50)
    x, w = codes(rng, (2, 5, 6, 3)), codes(rng, (4, 3, 3, 3))
    y = orc.conv3x3_fwd_f64(x, w)
    for b in range(2):
        for n in range(4):
            ref = sum(signal.correlate2d(x[b, :, :, c].astype(np.int64), w[n, :, :, c].astype(np.int64),
                                         mode="same", boundary="fill", fillvalue=0) for c in range(3))
            assert np.array_equal(y[b, :, :, n], ref)


def test_hand_worked_example():
    # 2x2 image of one channel, all-ones window: every output sees the whole image -> 1+2+3+4
    x = np.array([[[[1], [2]], [[3], [4]]]], dtype=np.int8)
    w = np.ones((1, 3, 3, 1), dtype=np.int8)
    assert np.array_equal(orc.conv3x3_fwd_f64(x, w).reshape(2, 2), [[10, 10], [10, 10]])
    # window that picks the upper-left neighbour only: output(h,w) = x(h-1,w-1), zero on the first row/column
    w = np.zeros((1, 3, 3, 1), dtype=np.int8); w[0, 0, 0, 0] = 1
    assert np.array_equal(orc.conv3x3_fwd_f64(x, w).reshape(2, 2), [[0, 0], [0, 1]])
    # its data gradient moves dY the other way: dX(h,w) = dY(h+1,w+1)
    dy = np.array([[[[5], [6]], [[7], [8]]]], dtype=np.int8)
    assert np.array_equal(orc.conv3x3_dgrad_f64(dy, w).reshape(2, 2), [[8, 0], [0, 0]])
    # and its weight gradient is sum dY(h,w) x(h-1,w-1) = 8*1 at tap (0,0), e.g. tap (1,1): 5+12+21+32
    x1 = x
    dw = orc.conv3x3_wgrad_f64(dy, x1).reshape(3, 3)
    assert dw[0, 0] == 8 and dw[1, 1] == 70 and dw[2, 2] == 5 * 4 and dw[0, 2] == 7 * 2 and dw[2, 0] == 6 * 3


@pytest.mark.parametrize("kh,kw", [(0, 0), (0, 2), (1, 1), (2, 1), (1, 0)])
def test_single_tap_kernels_are_shifts(kh, kw):
    rng = np.random.default_rng(51)
    x = codes(rng, (2, 4, 5, 3))
    w = np.zeros((3, 3, 3, 3), dtype=np.int8)
    for c in range(3):
        w[c, kh, kw, c] = 1
    y = orc.conv3x3_fwd_f64(x, w)
    want = np.zeros_like(y)
    for h in range(4):
        for v in range(5):
            hs, ws = h + kh - 1, v + kw - 1
            if 0 <= hs < 4 and 0 <= ws < 5:
                want[:, h, v, :] = x[:, hs, ws, :]
    assert np.array_equal(y, want)


def brute(x, w, dy):
    b, h, wd, c = x.shape
    n = w.shape[0]
    y = np.zeros((b, h, wd, n), dtype=object)
    dx = np.zeros((b, h, wd, c), dtype=object)
    dw = np.zeros((n, 3, 3, c), dtype=object)
    for bi in range(b):
        for hi in range(h):
            for wi in range(wd):
                for ni in range(n):
                    for kh in range(3):
                        for kw in range(3):
                            hs, ws = hi + kh - 1, wi + kw - 1
                            if not (0 <= hs < h and 0 <= ws < wd):
                                continue
                            for ci in range(c):
                                y[bi, hi, wi, ni] += int(x[bi, hs, ws, ci]) * int(w[ni, kh, kw, ci])
                                dx[bi, hs, ws, ci] += int(dy[bi, hi, wi, ni]) * int(w[ni, kh, kw, ci])
                                dw[ni, kh, kw, ci] += int(dy[bi, hi, wi, ni]) * int(x[bi, hs, ws, ci])
    return y, dx, dw


def test_against_brute_force_loops():
    rng = np.random.default_rng(52)
    x, w, dy = codes(rng, (2, 3, 4, 2)), codes(rng, (3, 3, 3, 2)), codes(rng, (2, 3, 4, 3))
    y, dx, dw = brute(x, w, dy)
    assert np.array_equal(orc.conv3x3_fwd_f64(x, w), y.astype(np.float64))
    assert np.array_equal(orc.conv3x3_dgrad_f64(dy, w), dx.astype(np.float64))
    assert np.array_equal(orc.conv3x3_wgrad_f64(dy, x), dw.astype(np.float64))


def test_adjoint_identities_exact():
    rng = np.random.default_rng(53)
    x, w, dy = codes(rng, (3, 6, 5, 4)), codes(rng, (5, 3, 3, 4)), codes(rng, (3, 6, 5, 5))
    lhs = int((orc.conv3x3_fwd_f64(x, w) * dy).sum())
    assert lhs == int((orc.conv3x3_dgrad_f64(dy, w) * x).sum())
    assert lhs == int((orc.conv3x3_wgrad_f64(dy, x) * w).sum())


def test_forward_and_wgrad_equal_the_patch_matrix_gemms():
    rng = np.random.default_rng(54)
    x, w, dy = codes(rng, (2, 7, 5, 16)), codes(rng, (8, 3, 3, 16)), codes(rng, (2, 7, 5, 8))
    patches = wl.im2col_nhwc_3x3(x)
    acc, _ = orc.int_gemm_nt(patches, w.reshape(8, 144))
    assert np.array_equal(orc.conv3x3_fwd_f64(x, w).reshape(-1, 8), acc)
    accw, _ = orc.int_gemm_nt(np.ascontiguousarray(dy.reshape(-1, 8).T), np.ascontiguousarray(patches.T))
    assert np.array_equal(orc.conv3x3_wgrad_f64(dy, x).reshape(8, 144), accw)


def test_dgrad_is_a_forward_convolution_with_flipped_transposed_weights():
    rng = np.random.default_rng(55)
    w, dy = codes(rng, (6, 3, 3, 4)), codes(rng, (2, 5, 7, 6))
    wflip = np.ascontiguousarray(w[:, ::-1, ::-1, :].transpose(3, 1, 2, 0))       # [C,3,3,N]: W'[c,a,b,n] = W[n,2-a,2-b,c]
    assert np.array_equal(orc.conv3x3_dgrad_f64(dy, w), orc.conv3x3_fwd_f64(dy, wflip))


def test_float_gradients_by_finite_differences():
    rng = np.random.default_rng(56)
    x, w = rng.standard_normal((1, 4, 3, 2)), rng.standard_normal((2, 3, 3, 2))
    dy = rng.standard_normal((1, 4, 3, 2))
    loss = lambda xx, ww: float((orc.conv3x3_fwd_f64(xx, ww) * dy).sum())
    dx, dw = orc.conv3x3_dgrad_f64(dy, w), orc.conv3x3_wgrad_f64(dy, x)
    eps = 1e-6
    for idx in [(0, 0, 0, 0), (0, 3, 2, 1), (0, 1, 1, 0)]:
        xp = x.copy(); xp[idx] += eps
        assert abs((loss(xp, w) - loss(x, w)) / eps - dx[idx]) < 1e-5
    for idx in [(0, 0, 0, 0), (1, 2, 2, 1), (1, 1, 0, 0)]:
        wp = w.copy(); wp[idx] += eps
        assert abs((loss(x, wp) - loss(x, w)) / eps - dw[idx]) < 1e-5


def test_operator_composition_matches_the_linear_operator_on_patches():
    """Forward and weight gradient of the convolution operator equal the linear operator on the patch matrix
    (same codes, same accumulators); the data gradient is the patch gradient folded back (col2im)."""
    rng = np.random.default_rng(57)
    act = np.abs(rng.standard_normal((2, 6, 5, 16))).astype(np.float16)
    w = (rng.standard_normal((8, 144)) * 0.1).astype(np.float32)
    dy = (rng.standard_normal((60, 8)) * 1e-3).astype(np.float16)
    bias = rng.standard_normal(8).astype(np.float32)
    for gran in ("tensor", "row"):
        cv = orc.conv3x3_operator_fwd_bwd(orc.INT8, act, w, bias, dy, gran, "stochastic", seed=9, offset=3)
        ln = orc.operator_fwd_bwd(orc.INT8, wl.im2col_nhwc_3x3(act), w, bias, dy, gran, "stochastic", seed=9, offset=3)
        assert np.array_equal(cv["acc"], ln["acc"]) and np.array_equal(cv["y"], ln["y"])
        assert np.array_equal(cv["dyq"], ln["dyq"]) and np.array_equal(cv["acc_dw"], ln["acc_dw"])
        assert np.array_equal(cv["dw"], ln["dw"])
        assert np.array_equal(wl.im2col_nhwc_3x3(cv["xq"].reshape(2, 6, 5, 16)), ln["xq"])
        if gran == "tensor":                      # same backward weight codes: fold the patch gradient
            patch_grad = ln["acc_dx"].astype(np.int64).reshape(2, 6, 5, 3, 3, 16)
            fold = np.zeros((2, 8, 7, 16), dtype=np.int64)
            for kh in range(3):
                for kw in range(3):
                    fold[:, kh:kh + 6, kw:kw + 5, :] += patch_grad[:, :, :, kh, kw, :]
            assert np.array_equal(cv["acc_dx"].reshape(2, 6, 5, 16), fold[:, 1:7, 1:6, :])
        else:                                     # per-input-channel scales: one per c, shared by all taps
            assert cv["swb"].shape == (16,)
            w9 = w.reshape(72, 16)
            assert np.array_equal(cv["swb"], (np.abs(w9).max(axis=0) / np.float32(127)).astype(np.float32))


def test_against_torch_conv2d_and_its_autograd():
    """An independent library: torch's CPU convolution in double and the gradients its autograd derives."""
    import torch
    rng = np.random.default_rng(58)
    x = rng.integers(-127, 128, (2, 6, 7, 5)).astype(np.float64)          # NHWC
    w = rng.integers(-127, 128, (4, 3, 3, 5)).astype(np.float64)          # [N, kh, kw, C]
    dy = rng.integers(-127, 128, (2, 6, 7, 4)).astype(np.float64)
    xt = torch.tensor(x.transpose(0, 3, 1, 2).copy(), requires_grad=True)          # NCHW
    wt = torch.tensor(w.transpose(0, 3, 1, 2).copy(), requires_grad=True)          # [N, C, kh, kw]
    yt = torch.nn.functional.conv2d(xt, wt, padding=1)
    yt.backward(torch.tensor(dy.transpose(0, 3, 1, 2).copy()))
    assert np.array_equal(orc.conv3x3_fwd_f64(x, w), yt.detach().numpy().transpose(0, 2, 3, 1))
    assert np.array_equal(orc.conv3x3_dgrad_f64(dy, w), xt.grad.numpy().transpose(0, 2, 3, 1))
    assert np.array_equal(orc.conv3x3_wgrad_f64(dy, x), wt.grad.numpy().transpose(0, 2, 3, 1))
