"""3x3 NHWC convolution as implicit GEMM against the CPU oracle (GPU, through the C ABI).

Integer accumulators are compared bit for bit, dequantized outputs within rtol 1e-3 and
atol 1e-3 * max|want| (fp16 outputs add half an ulp of binary16).
"""
import numpy as np
import pytest
import torch

from oracle import qsync_oracle as orc
from paper_2407_02327_amd import qsync as Q
from paper_2407_02327_amd import workloads as wl
from paper_2407_02327_amd.operator import QConv3x3
from tests.gpu_util import GRAN, RND, assert_bits_equal, assert_close, dev, empty, host, say

pytestmark = pytest.mark.gpu

SHAPES = [(1, 4, 4, 16, 8), (2, 7, 5, 16, 24), (3, 8, 8, 64, 64), (1, 13, 16, 48, 40), (1, 9, 9, 128, 72),
          (1, 6, 6, 256, 32), (2, 33, 17, 32, 136), (1, 3, 70, 80, 260)]


@pytest.fixture(autouse=True)
def planner_choice_restored():
    yield
    Q.qsync_debug_set_gemm_tile(-1)


@pytest.mark.parametrize("tile", [-1, 0, 1, 2])
def test_implicit_gemm_on_codes_bit_exact(tile):
    rng = np.random.default_rng(60)
    Q.qsync_debug_set_gemm_tile(tile)
    for (b, h, w, c, n) in SHAPES:
        say("conv codes", "tile", tile, b, h, w, c, n)
        xq = rng.integers(-127, 128, (b, h, w, c)).astype(np.int8)
        wq = rng.integers(-127, 128, (n, 9 * c)).astype(np.int8)
        sx = np.array([0.01], np.float32)
        sw = (rng.random(n) * 0.02 + 0.001).astype(np.float32)
        bias = rng.standard_normal(n).astype(np.float32)
        want_acc = orc.conv3x3_fwd_f64(xq, wq.reshape(n, 3, 3, c)).reshape(-1, n)
        want_y = want_acc * float(sx[0]) * sw.astype(np.float64).reshape(1, -1) + bias.astype(np.float64)
        M = b * h * w
        acc, y = empty((M, n), torch.int32), empty((M, n), torch.float32)
        Q.qsync_conv3x3_fwd(Q.INT8, b, h, w, c, n, dev(xq), dev(sx), dev(wq), dev(sw), Q.PER_ROW, dev(bias), y, acc)
        assert_bits_equal(host(acc), want_acc.astype(np.int32), "accumulators")
        assert_close(host(y), want_y, "Y with accumulator dump")
        for ydt in (torch.float32, torch.float16):              # the vectorized epilogue (no dump)
            y2 = empty((M, n), ydt)
            Q.qsync_conv3x3_fwd(Q.INT8, b, h, w, c, n, dev(xq), dev(sx), dev(wq), dev(sw), Q.PER_ROW, dev(bias), y2)
            assert_close(host(y2), want_y, f"Y {ydt}")
        st = np.array([0.5], np.float32)                        # per-tensor weight scale, no bias
        Q.qsync_conv3x3_fwd(Q.INT8, b, h, w, c, n, dev(xq), dev(sx), dev(wq), dev(st), Q.PER_TENSOR, None, y)
        assert_close(host(y), want_acc * float(sx[0]) * 0.5, "Y per-tensor")


@pytest.mark.parametrize("tile", [-1, 0, 2])
def test_implicit_gemm_fp16(tile):
    rng = np.random.default_rng(61)
    Q.qsync_debug_set_gemm_tile(tile)
    for (b, h, w, c, n) in [(2, 7, 5, 8, 24), (3, 8, 8, 64, 64), (1, 13, 16, 40, 40), (1, 6, 6, 256, 32)]:
        say("conv fp16", "tile", tile, b, h, w, c, n)
        x = rng.standard_normal((b, h, w, c)).astype(np.float16)
        wt = (rng.standard_normal((n, 9 * c)) * 0.05).astype(np.float16)
        bias = rng.standard_normal(n).astype(np.float32)
        want = orc.conv3x3_fwd_f64(x, wt.reshape(n, 3, 3, c)).reshape(-1, n) + bias.astype(np.float64)
        y = empty((b * h * w, n), torch.float32)
        Q.qsync_conv3x3_fwd(Q.FP16, b, h, w, c, n, dev(x), None, dev(wt), None, Q.PER_TENSOR, dev(bias), y)
        assert_close(host(y), want, "Y fp16 tag")


def test_weight_flip_bit_exact():
    rng = np.random.default_rng(62)
    for (n, c) in [(8, 16), (64, 64), (5, 3), (136, 32)]:
        w = rng.integers(-127, 128, (n, 3, 3, c)).astype(np.int8)
        want = np.ascontiguousarray(w[:, ::-1, ::-1, :].transpose(3, 1, 2, 0)).reshape(c, 9 * n)
        out = empty((c, 9 * n), torch.int8)
        Q.qsync_conv3x3_wflip(dev(w.reshape(n, 9 * c)), n, c, out)
        assert_bits_equal(host(out), want, "flipped codes")
        wh = rng.standard_normal((n, 3, 3, c)).astype(np.float16)
        outh = empty((c, 9 * n), torch.float16)
        Q.qsync_conv3x3_wflip(dev(wh.reshape(n, 9 * c)), n, c, outh)
        assert_bits_equal(host(outh), np.ascontiguousarray(wh[:, ::-1, ::-1, :].transpose(3, 1, 2, 0)).reshape(c, 9 * n), "flipped halves")


@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_conv_prepare_weights_equals_the_separate_calls(dt):
    rng = np.random.default_rng(66)
    for (n, c) in [(64, 64), (8, 16), (24, 48), (136, 32), (256, 128), (5, 3), (48, 80), (32, 16)]:   # N % 16 != 0: separate passes
        say("conv weights", dt.__name__, n, c)
        w = (rng.standard_normal((n, 9 * c)) * 0.05).astype(dt)
        w[:, c - 1::c] = 0                              # an all-zero input channel: scale 1
        e = lambda *s_, t=torch.float32: empty(tuple(s_), t)
        sw, iw, swb, iwb = e(n), e(n), e(c), e(c)
        wq, wflip = e(n, 9 * c, t=torch.int8), e(c, 9 * n, t=torch.int8)
        from tests.gpu_util import ws
        Q.qsync_conv3x3_prepare_weights(dev(w), n, c, 8, sw, iw, wq, swb, iwb, wflip,
                                        ws(Q.qsync_conv3x3_prepare_weights_workspace_bytes(n, c)))
        sr, ir = orc.scales_from_amax(orc.absmax(w, "row"))
        w9 = w.reshape(9 * n, c)
        sc, ic = orc.scales_from_amax(orc.absmax(w9, "col"))
        assert_bits_equal(host(sw), sr, "per-n scales")
        assert_bits_equal(host(iw), ir, "per-n inverse scales")
        assert_bits_equal(host(swb), sc, "per-c scales")
        assert_bits_equal(host(iwb), ic, "per-c inverse scales")
        assert_bits_equal(host(wq), orc.quantize_int(w, ir, "row", "nearest"), "forward codes")
        wqb = orc.quantize_int(w9, ic, "col", "nearest").reshape(n, 3, 3, c)
        assert_bits_equal(host(wflip), np.ascontiguousarray(wqb[:, ::-1, ::-1, :].transpose(3, 1, 2, 0)).reshape(c, 9 * n),
                          "mirrored backward codes")


@pytest.mark.parametrize("tile", [-1, 0, 1, 2])
def test_weight_gradient_on_codes_bit_exact(tile):
    from tests.gpu_util import ws
    rng = np.random.default_rng(67)
    Q.qsync_debug_set_gemm_tile(tile)
    # (pixel counts that are multiples of 128 take the gathering TN GEMM, the others the padded transposed copies)
    for (b, h, w, c, n) in [(1, 4, 4, 16, 16), (2, 7, 5, 16, 32), (3, 8, 8, 64, 64), (1, 13, 16, 48, 48), (2, 3, 70, 80, 16),
                            (5, 9, 15, 32, 144), (1, 1, 1, 16, 16), (2, 31, 33, 16, 16),
                            (2, 8, 8, 16, 16), (4, 8, 8, 64, 64), (2, 16, 16, 48, 48), (8, 4, 4, 80, 16), (1, 16, 24, 32, 144),
                            (128, 1, 1, 16, 16), (4, 32, 32, 64, 64), (64, 2, 3, 16, 32), (16, 28, 28, 128, 256)]:
        say("conv wgrad codes", "tile", tile, b, h, w, c, n)
        xq = rng.integers(-127, 128, (b, h, w, c)).astype(np.int8)
        dyq = rng.integers(-127, 128, (b, h, w, n)).astype(np.int8)
        sx, sdy = np.array([0.02], np.float32), np.array([3e-4], np.float32)
        want_acc = orc.conv3x3_wgrad_f64(dyq, xq).reshape(n, 9 * c)
        acc, dw = empty((n, 9 * c), torch.int32), empty((n, 9 * c), torch.float32)
        wsp = ws(Q.qsync_conv3x3_wgrad_workspace_bytes(Q.INT8, b, h, w, c, n))
        wsp.fill_(0x5A)                                           # nothing in the workspace needs initialising
        Q.qsync_conv3x3_wgrad(Q.INT8, b, h, w, c, n, dev(xq), dev(sx), dev(dyq.reshape(-1, n)), dev(sdy), dw, acc, wsp)
        assert_bits_equal(host(acc), want_acc.astype(np.int32), "weight-gradient accumulators")
        assert_close(host(dw), want_acc * float(sx[0]) * float(sdy[0]), "dW with accumulator dump")
        dwh = empty((n, 9 * c), torch.float16)
        Q.qsync_conv3x3_wgrad(Q.INT8, b, h, w, c, n, dev(xq), dev(sx), dev(dyq.reshape(-1, n)), dev(sdy), dwh, None, wsp)
        assert_close(host(dwh), want_acc * float(sx[0]) * float(sdy[0]), "dW fp16")


@pytest.mark.parametrize("tile", [-1, 0, 2])
def test_weight_gradient_fp16(tile):
    from tests.gpu_util import ws
    rng = np.random.default_rng(69)
    Q.qsync_debug_set_gemm_tile(tile)
    for (b, h, w, c, n) in [(1, 4, 4, 8, 8), (2, 7, 5, 16, 24), (3, 8, 8, 64, 64), (1, 13, 16, 40, 48), (2, 3, 70, 8, 16),
                            (1, 1, 1, 8, 8), (2, 31, 33, 16, 8),
                            (2, 8, 8, 8, 8), (4, 8, 8, 64, 64), (2, 16, 16, 40, 48), (1, 16, 24, 32, 136), (128, 1, 1, 8, 8),
                            (4, 32, 32, 64, 64), (64, 2, 3, 16, 24)]:
        say("conv wgrad fp16", "tile", tile, b, h, w, c, n)
        x = rng.standard_normal((b, h, w, c)).astype(np.float16)
        dy = (rng.standard_normal((b, h, w, n)) * 0.05).astype(np.float16)
        want = orc.conv3x3_wgrad_f64(dy, x).reshape(n, 9 * c)
        dw = empty((n, 9 * c), torch.float32)
        wsp = ws(Q.qsync_conv3x3_wgrad_workspace_bytes(Q.FP16, b, h, w, c, n))
        wsp.fill_(0xFF)                                           # uninitialised workspace full of NaN patterns
        Q.qsync_conv3x3_wgrad(Q.FP16, b, h, w, c, n, dev(x), None, dev(dy.reshape(-1, n)), None, dw, None, wsp)
        assert_close(host(dw), want, "dW fp16 tag")


def conv_case(batch, hh, ww, c, n, seed):
    rng = np.random.default_rng(seed)
    act = np.abs(rng.standard_normal((batch, hh, ww, c))).astype(np.float16)
    w = (rng.standard_normal((n, 9 * c)) * np.sqrt(2.0 / (9 * c))).astype(np.float32)
    dy = (rng.standard_normal((batch * hh * ww, n)) * 1e-3).astype(np.float16)
    bias = rng.standard_normal(n).astype(np.float32)
    return act, w, bias, dy


def run_conv_operator(act, w, bias, dy, w_gran, dy_round="stochastic", seed=5, via_patches=False):
    b, h, wd, c = act.shape
    n = w.shape[0]
    op = QConv3x3(Q.INT8, b, h, wd, c, n, x_dtype=torch.float16, y_dtype=torch.float32, dx_dtype=torch.float16,
                  w_gran=GRAN[w_gran], dy_round=RND[dy_round], philox_seed=seed, dump_acc=True,
                  wgrad_via_patches=via_patches)
    op.bias.copy_(dev(bias))
    op.forward(dev(act), dev(w))
    op.backward(dev(dy))
    ref = orc.conv3x3_operator_fwd_bwd(orc.INT8, act, w, bias, dy, w_gran, dy_round, seed=seed, offset=0,
                                       y_dtype=np.float64, dx_dtype=np.float64, dw_dtype=np.float64)
    assert_bits_equal(host(op.sx), ref["sx"], "sx")
    assert_bits_equal(host(op.sw), ref["sw"], "sw")
    assert_bits_equal(host(op.xq), ref["xq"], "xq")
    assert_bits_equal(host(op.wq), ref["wq"], "wq")
    assert_bits_equal(host(op.acc), ref["acc"], "forward accumulators")
    assert_close(host(op.y), ref["y"], "Y")
    assert_bits_equal(host(op.sdy), ref["sdy"], "sdy")
    assert_bits_equal(host(op.dyq), ref["dyq"], "dyq")
    assert_bits_equal(host(op.swb), ref["swb"], "swb")
    flipped = np.ascontiguousarray(ref["wqb"].reshape(n, 3, 3, c)[:, ::-1, ::-1, :].transpose(3, 1, 2, 0)).reshape(c, 9 * n)
    assert_bits_equal(host(op.wflip), flipped, "mirrored backward codes")
    assert_bits_equal(host(op.acc_dx), ref["acc_dx"], "dgrad accumulators")
    assert_bits_equal(host(op.acc_dw), ref["acc_dw"], "wgrad accumulators")
    assert_close(host(op.dx), ref["dx"], "dX")
    assert_close(host(op.dw), ref["dw"], "dW")
    assert_close(host(op.db), ref["db"], "db")
    assert not ref["overflow"]
    return op


@pytest.mark.parametrize("w_gran", ["row", "tensor"])
def test_conv_operator_small(w_gran):
    run_conv_operator(*conv_case(2, 12, 8, 16, 32, 63), w_gran)
    run_conv_operator(*conv_case(1, 16, 16, 64, 32, 64), w_gran, dy_round="nearest")
    run_conv_operator(*conv_case(2, 12, 8, 16, 32, 68), w_gran, via_patches=True)


def test_conv_operator_fp16_forward_and_dgrad():
    act, w, bias, dy = conv_case(2, 12, 8, 16, 24, 65)
    op = QConv3x3(Q.FP16, 2, 12, 8, 16, 24, x_dtype=torch.float16, y_dtype=torch.float32, dx_dtype=torch.float32)
    op.bias.copy_(dev(bias))
    op.forward(dev(act), dev(w))
    op.backward(dev(dy))
    ref = orc.conv3x3_operator_fwd_bwd(orc.FP16, act, w, bias, dy, y_dtype=np.float64, dx_dtype=np.float64,
                                       dw_dtype=np.float64)
    assert_bits_equal(host(op.wq), ref["wq"], "cast weights")
    assert_close(host(op.y), ref["y"], "Y")
    assert_close(host(op.dx), ref["dx"], "dX")
    assert_close(host(op.dw), ref["dw"], "dW")


def test_config3_resnet_conv_implicit_full_size_fp16_tag():
    """Config 3 as a convolution with the FP16 precision tag at full size: implicit forward and data gradient,
    weight gradient over the padded pixel axis."""
    case = wl.config3()
    b, h, wd, c = case.nhwc.shape
    n = case.w.shape[0]
    say("config3 conv fp16 tag full size")
    op = QConv3x3(Q.FP16, b, h, wd, c, n, x_dtype=torch.float16, y_dtype=torch.float16, dx_dtype=torch.float16)
    op.bias.copy_(dev(case.bias))
    op.forward(dev(case.nhwc), dev(case.w))
    op.backward(dev(case.dy))
    ref = orc.conv3x3_operator_fwd_bwd(orc.FP16, case.nhwc, case.w, case.bias, case.dy, y_dtype=np.float64,
                                       dx_dtype=np.float64, dw_dtype=np.float64)
    assert_bits_equal(host(op.wq), ref["wq"], "cast weights")
    assert_close(host(op.y), ref["y"], "Y")
    assert_close(host(op.dx), ref["dx"], "dX")
    assert_close(host(op.dw), ref["dw"], "dW")


def test_config3_resnet_conv_implicit_full_size():
    case = wl.config3()
    run_conv_operator(case.nhwc, case.w, case.bias, case.dy, case.w_gran, case.dy_round, seed=case.philox_seed)


@pytest.mark.parametrize("tile", [-1, 1])
def test_chained_convolution_takes_its_scale_from_the_producers_epilogue(tile):
    """Two convolutions back to back: the producer's forward collects max |Y| where it stores Y
    (qsync_conv3x3_fwd_amax), the consumer forms its activation scale from that word and quantizes Y without a
    maximum pass of its own.  Y of the producer is unchanged bit for bit; scale, codes and accumulators of the
    consumer equal those of a consumer that finds the maximum itself, and the oracle's on the same Y; the consumed
    maximum starts the next step at zero."""
    Q.qsync_debug_set_gemm_tile(tile)
    try:
        rng = np.random.default_rng(31)
        b, h, w, c0, c1, c2 = 2, 12, 10, 32, 48, 16
        act = np.abs(rng.standard_normal((b, h, w, c0))).astype(np.float16)
        w0 = (rng.standard_normal((c1, 9 * c0)) * np.sqrt(2.0 / (9 * c0))).astype(np.float32)
        w1 = (rng.standard_normal((c2, 9 * c1)) * np.sqrt(2.0 / (9 * c1))).astype(np.float32)
        kw = dict(x_dtype=torch.float16, y_dtype=torch.float16)
        prod = QConv3x3(Q.INT8, b, h, w, c0, c1, collect_y_amax=True, **kw)
        plain = QConv3x3(Q.INT8, b, h, w, c0, c1, **kw)
        cons = QConv3x3(Q.INT8, b, h, w, c1, c2, dump_acc=True, **kw)
        base = QConv3x3(Q.INT8, b, h, w, c1, c2, dump_acc=True, **kw)
        for step in range(2):
            y0 = prod.forward(dev(act), dev(w0))
            y0_plain = plain.forward(dev(act), dev(w0))
            cons.forward(y0.view(b, h, w, c1), dev(w1), x_amax=prod.y_amax)
            base.forward(y0.view(b, h, w, c1), dev(w1))
            torch.cuda.synchronize()
            assert torch.equal(y0, y0_plain), step
            assert prod.y_amax.item() == 0.0
            for name in ("sx", "ix", "xq", "acc", "y"):
                assert torch.equal(getattr(cons, name), getattr(base, name)), (step, name)
        y0h = host(y0).reshape(b, h, w, c1)
        amax = np.abs(y0h.astype(np.float32)).max()
        s_ref, i_ref = orc.scales_from_amax(np.array([amax], np.float32))
        assert_bits_equal(host(cons.sx), s_ref, "consumer scale")
        xq_ref = orc.quantize_int(y0h.reshape(-1, c1), i_ref, "tensor", "nearest")
        assert_bits_equal(host(cons.xq), xq_ref, "consumer codes")
        wq = host(cons.wq).reshape(c2, 3, 3, c1)
        want_acc = orc.conv3x3_fwd_f64(xq_ref.reshape(b, h, w, c1), wq).reshape(-1, c2)
        assert_bits_equal(host(cons.acc), want_acc.astype(np.int32), "consumer accumulators")
    finally:
        Q.qsync_debug_set_gemm_tile(-1)
