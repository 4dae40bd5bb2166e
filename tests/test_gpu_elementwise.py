"""GPU parity: absmax/scale, quantize, cast, dequantize against the CPU oracle, element by element.

Integer codes, scales (one IEEE division each) and casts must match bit for bit; dequantized
values are held to rtol 1e-3 / atol 1e-3*max|y|.
"""
import numpy as np
import pytest
import torch

from oracle import qsync_oracle as orc
from paper_2407_02327_amd import qsync as Q
from tests.gpu_util import GRAN, RND, assert_bits_equal, assert_close, dev, empty, host, say, ws

pytestmark = pytest.mark.gpu
TORCH = {np.float32: torch.float32, np.float16: torch.float16}


def _data(rng, shape, dtype, sigma=1.0):
    x = (rng.standard_normal(shape) * sigma).astype(dtype)
    return x


def _gpu_absmax(xd, rows, cols, ld, gran, bits=8):
    n = {"tensor": 1, "row": rows, "col": cols}[gran]
    s, iv, am = empty(n, torch.float32), empty(n, torch.float32), empty(n, torch.float32)
    w = ws(Q.qsync_absmax_workspace_bytes(rows, cols, GRAN[gran]))
    Q.qsync_absmax_scale(xd, rows, cols, ld, GRAN[gran], bits, s, iv, am, None, w)
    return s, iv, am


SHAPES = [(1, 1), (3, 5), (64, 128), (130, 72), (257, 1000), (512, 4096), (1000, 24), (33, 8200)]


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("gran", ["tensor", "row", "col"])
def test_absmax_scale(dtype, gran):
    rng = np.random.default_rng(1)
    for rows, cols in SHAPES:
        for bits in (8, 4):
            say("absmax", dtype.__name__, gran, rows, cols, bits)
            x = _data(rng, (rows, cols), dtype, 3.0)
            if rows > 2:
                x[1, :] = 0                                   # an all-zero row
            s, iv, am = _gpu_absmax(dev(x), rows, cols, cols, gran, bits)
            amax = orc.absmax(x, gran)
            so, io = orc.scales_from_amax(amax, bits)
            assert_bits_equal(host(am), amax, "amax")
            assert_bits_equal(host(s), so, "scale")
            assert_bits_equal(host(iv), io, "inv_scale")


def test_absmax_strided_and_misaligned_and_zero():
    rng = np.random.default_rng(2)
    big = _data(rng, (70, 200), np.float32)
    bd = dev(big)
    for gran in ("tensor", "row", "col"):
        say("absmax strided", gran)
        view = bd[:, 3:3 + 150]                               # ld 200, base offset 12 bytes
        s, iv, am = _gpu_absmax(view, 70, 150, 200, gran)
        assert_bits_equal(host(am), orc.absmax(big[:, 3:153], gran), "amax strided")
    z = np.zeros((16, 64), np.float16)
    s, iv, am = _gpu_absmax(dev(z), 16, 64, 64, "tensor")
    assert host(s)[0] == 1 and host(iv)[0] == 1 and host(am)[0] == 0
    # large tensor: every stage-1 block is used
    say("absmax large")
    x = _data(rng, (4096, 4096), np.float16)
    x[4095, 4095] = 77.0
    s, iv, am = _gpu_absmax(dev(x), 4096, 4096, 4096, "tensor")
    assert host(am)[0] == 77.0


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_absmax_fused_with_column_sums(dtype):
    """One pass gives the per-tensor scale and the column sums (the bias gradient when x = dY)."""
    rng = np.random.default_rng(7)
    for rows, cols in [(1, 1), (3, 5), (64, 128), (257, 1000), (4096, 512), (2000, 24), (33, 8200), (16384, 64)]:
        say("absmax+colsum", dtype.__name__, rows, cols)
        x = _data(rng, (rows, cols), dtype, 1e-2)
        xd = dev(x)
        s, iv, am, cs = (empty(1, torch.float32), empty(1, torch.float32), empty(1, torch.float32),
                         empty(cols, torch.float32))
        w = ws(Q.qsync_absmax_workspace_bytes(rows, cols, Q.PER_TENSOR))
        Q.qsync_absmax_scale(xd, rows, cols, cols, Q.PER_TENSOR, 8, s, iv, am, cs, w)
        amax = orc.absmax(x, "tensor")
        so, io = orc.scales_from_amax(amax)
        assert_bits_equal(host(am), amax, "amax")
        assert_bits_equal(host(s), so, "scale")
        assert_bits_equal(host(iv), io, "inv_scale")
        assert_close(host(cs), x.astype(np.float64).sum(axis=0), "column sums")
    with pytest.raises(Q.QsyncError) as e:
        Q.qsync_absmax_scale(xd, rows, cols, cols, Q.PER_ROW, 8, s, iv, am, cs, w)
    assert e.value.status == Q.ERR_UNSUPPORTED


@pytest.mark.parametrize("k", [10, 9, 7])
def test_fp16_stochastic_cast_bit_exact(k):
    """Floating-point stochastic quantization to binary16: same draws, same integer decision, same bits."""
    rng = np.random.default_rng(31)
    for rows, cols in [(1, 1), (5, 7), (64, 64), (130, 72), (257, 1000), (1024, 768)]:
        say("fp16 SR cast", k, rows, cols)
        x = (rng.standard_normal((rows, cols)) * np.exp(rng.uniform(-14, 9, (rows, cols)))).astype(np.float32)
        if rows * cols > 16:
            x.reshape(-1)[:8] = [0.0, -0.0, 65504.0, 65530.0, 2.0 ** -24, -2.0 ** -26, 1.0, 2.0 - 2.0 ** -12]
        xd = dev(x)
        q, qt = empty((rows, cols), torch.float16), empty((cols, rows), torch.float16)
        Q.qsync_quantize(xd, rows, cols, cols, Q.FP16, k, 0, Q.ROUND_STOCHASTIC, 99, 4242, None, q, qt)
        want = orc.cast_fp16_stochastic(x, seed=99, offset=4242, k=k)
        assert_bits_equal(host(q).view(np.uint16), want.view(np.uint16), "fp16 SR")
        assert_bits_equal(host(qt).view(np.uint16), np.ascontiguousarray(want.T).view(np.uint16), "fp16 SR transposed")
    with pytest.raises(Q.QsyncError) as e:
        Q.qsync_quantize(xd, rows, cols, cols, Q.FP16, 5, 0, Q.ROUND_STOCHASTIC, 1, 0, None, q, qt)
    assert e.value.status == Q.ERR_UNSUPPORTED
    # binary16 input: a copy whatever the rounding mode
    h = x.astype(np.float16)
    Q.qsync_quantize(dev(h), rows, cols, cols, Q.FP16, 0, 0, Q.ROUND_STOCHASTIC, 1, 0, None, q, None)
    assert_bits_equal(host(q).view(np.uint16), h.view(np.uint16), "fp16 copy")


@pytest.mark.parametrize("dt", [np.float32, np.float16])
def test_prepare_weights_equals_the_separate_calls(dt):
    """Fused weight preparation (row and column maxima in one pass, both sets of codes in another) against the
    oracle's per-row and per-column quantizations; shapes on the fused path (both row-group sizes) and off it."""
    rng = np.random.default_rng(42)
    for (n, k) in [(64, 576), (1024, 4096), (4096, 1024), (3072, 768), (48, 40), (20, 24), (16, 8), (8208, 64)]:
        say("prepare weights", dt.__name__, n, k)
        w = (rng.standard_normal((n, k)) * 0.02).astype(dt)
        w[rng.integers(0, n), :] = 0                       # an all-zero row: scale 1
        sw, iw, aw = empty((n,), torch.float32), empty((n,), torch.float32), empty((n,), torch.float32)
        swb, iwb = empty((k,), torch.float32), empty((k,), torch.float32)
        wq, wqbT = empty((n, k), torch.int8), empty((k, n), torch.int8)
        Q.qsync_prepare_weights(dev(w), n, k, 8, sw, iw, aw, wq, swb, iwb, wqbT, ws(Q.qsync_absmax_workspace_bytes(n, k, Q.PER_COL)))
        ar, ac = orc.absmax(w, "row"), orc.absmax(w, "col")
        sr, ir = orc.scales_from_amax(ar)
        sc, ic = orc.scales_from_amax(ac)
        assert_bits_equal(host(aw), ar, "row maxima")
        assert_bits_equal(host(sw), sr, "row scales")
        assert_bits_equal(host(iw), ir, "row inverse scales")
        assert_bits_equal(host(swb), sc, "column scales")
        assert_bits_equal(host(iwb), ic, "column inverse scales")
        assert_bits_equal(host(wq), orc.quantize_int(w, ir, "row", "nearest"), "row-scaled codes")
        assert_bits_equal(host(wqbT), orc.quantize_int(w, ic, "col", "nearest").T, "column-scaled codes, transposed")


def test_im2col_on_codes_bit_exact():
    from paper_2407_02327_amd import workloads as wl
    rng = np.random.default_rng(41)
    for (b, h, w, c) in [(1, 4, 4, 16), (2, 7, 5, 16), (3, 8, 8, 64), (2, 56, 56, 64), (1, 13, 16, 48)]:
        say("im2col codes", b, h, w, c)
        xq = rng.integers(-127, 128, (b, h, w, c)).astype(np.int8)
        M, K = b * h * w, 9 * c
        want = wl.im2col_nhwc_3x3(xq)
        a = empty((M, K), torch.int8); a.fill_(5)
        aT = None
        if M % 16 == 0:
            aT = empty((K, M), torch.int8); aT.fill_(5)
        Q.qsync_im2col3x3_i8(dev(xq), b, h, w, c, a, aT)
        assert_bits_equal(host(a), want, "patch matrix")
        if aT is not None:
            assert_bits_equal(host(aT), np.ascontiguousarray(want.T), "transposed patch matrix")
            a2 = empty((K, M), torch.int8)
            Q.qsync_im2col3x3_i8(dev(xq), b, h, w, c, None, a2)            # transposed copy alone
            assert_bits_equal(host(a2), np.ascontiguousarray(want.T), "transposed patch matrix alone")


def test_absmax_workspace_is_reusable_without_clearing():
    """The arrival counters at the start of the workspace are zeroed once by the caller and left zero
    by every call: one buffer serves a sequence of different reductions, each checked against the oracle."""
    rng = np.random.default_rng(11)
    shapes = [(4096, 4096), (64, 128), (16384, 1024), (257, 1000), (8192, 72), (33, 8200), (3, 5), (4096, 4096)]
    nbytes = max(max(Q.qsync_absmax_workspace_bytes(r, c, Q.PER_TENSOR), Q.qsync_absmax_workspace_bytes(r, c, Q.PER_COL))
                 for r, c in shapes)
    w = ws(nbytes)
    for rep, (rows, cols) in enumerate(shapes):
        dtype = np.float16 if rep % 2 == 0 else np.float32
        x = _data(rng, (rows, cols), dtype, 0.5)
        xd = dev(x)
        for gran, with_sums in (("tensor", False), ("col", False), ("tensor", True)):
            say("absmax reuse", rows, cols, dtype.__name__, gran, with_sums)
            n = 1 if gran == "tensor" else cols
            sc, iv, am = empty(n, torch.float32), empty(n, torch.float32), empty(n, torch.float32)
            cs = empty(cols, torch.float32) if with_sums else None
            Q.qsync_absmax_scale(xd, rows, cols, cols, GRAN[gran], 8, sc, iv, am, cs, w)
            amax = orc.absmax(x, gran)
            so, io = orc.scales_from_amax(amax)
            assert_bits_equal(host(am), amax, "amax")
            assert_bits_equal(host(sc), so, "scale")
            assert_bits_equal(host(iv), io, "inv_scale")
            if with_sums:
                assert_close(host(cs), x.astype(np.float64).sum(axis=0), "column sums")
    assert int(w[:256].to(torch.int32).abs().sum().item()) == 0, "the arrival counter must be left at zero"


def test_absmax_column_sums_are_reproducible():
    """The in-kernel fold uses a fixed assignment and order: two runs give identical bits."""
    rng = np.random.default_rng(12)
    rows, cols = 16384, 4096
    xd = dev(_data(rng, (rows, cols), np.float16, 1e-2))
    w = ws(Q.qsync_absmax_workspace_bytes(rows, cols, Q.PER_TENSOR))
    outs = []
    for _ in range(3):
        sc, iv, am, cs = (empty(1, torch.float32), empty(1, torch.float32), empty(1, torch.float32),
                          empty(cols, torch.float32))
        Q.qsync_absmax_scale(xd, rows, cols, cols, Q.PER_TENSOR, 8, sc, iv, am, cs, w)
        outs.append((host(cs).copy(), host(sc).copy()))
    for cs, sc in outs[1:]:
        assert_bits_equal(cs, outs[0][0], "column sums, repeated run")
        assert_bits_equal(sc, outs[0][1], "scale, repeated run")


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_absmax_with_squared_norm(dtype):
    """The indicator statistics: one pass yields the scale, the squared norm and (optionally) the column sums."""
    rng = np.random.default_rng(13)
    for rows, cols in [(1, 1), (3, 5), (64, 128), (257, 1000), (4096, 512), (33, 8200), (16384, 1024)]:
        for with_sums in (False, True):
            say("absmax+sumsq", dtype.__name__, rows, cols, with_sums)
            x = _data(rng, (rows, cols), dtype, 0.7)
            xd = dev(x)
            sc, iv, am, sq = (empty(1, torch.float32) for _ in range(4))
            cs = empty(cols, torch.float32) if with_sums else None
            w = ws(Q.qsync_absmax_workspace_bytes(rows, cols, Q.PER_TENSOR))
            Q.qsync_absmax_scale(xd, rows, cols, cols, Q.PER_TENSOR, 8, sc, iv, am, cs, w, sumsq_opt=sq)
            st = orc.tensor_stats(x)
            assert_bits_equal(host(am), orc.absmax(x, "tensor"), "amax")
            assert_bits_equal(host(sc), orc.scales_from_amax(orc.absmax(x, "tensor"))[0], "scale")
            assert abs(float(host(sq)[0]) - st["sumsq"]) <= 1e-4 * st["sumsq"] + 1e-30, (float(host(sq)[0]), st["sumsq"])
            if with_sums:
                assert_close(host(cs), x.astype(np.float64).sum(axis=0), "column sums")


def test_indicator_from_device_statistics_matches_oracle():
    from paper_2407_02327_amd import indicator as ind
    rng = np.random.default_rng(14)
    w = (rng.standard_normal((768, 512)) * 0.02).astype(np.float32)
    v = rng.standard_normal((2048, 512)).astype(np.float16)
    g = (rng.standard_normal((2048, 768)) * 1e-3).astype(np.float16)
    sw, sv, sg = ind.tensor_stats(dev(w)), ind.tensor_stats(dev(v)), ind.tensor_stats(dev(g))
    ow, ov, og = orc.tensor_stats(w), orc.tensor_stats(v), orc.tensor_stats(g)
    for got, want in ((sw, ow), (sv, ov), (sg, og)):
        assert got.amax == want["amax"] and got.D == want["D"]
        assert abs(got.sumsq - want["sumsq"]) <= 1e-4 * want["sumsq"]
    q_x, q_v = ow["amax"] / 127, ov["amax"] / 127
    for kind in ("fixed", "float"):
        a = ind.variance_increment(kind, sw, sv, sg, q_x=q_x, q_v=q_v, k=9, gamma=1.5, d_o=3, d_L=24)
        b = orc.variance_increment(kind, ow, ov, og, q_x=q_x, q_v=q_v, eps=2.0 ** -9, gamma=1.5, d_o=3, d_L=24)
        for k in ("sigma_fp", "sigma_bp", "omega"):
            assert a[k] == pytest.approx(b[k], rel=2e-4), (kind, k)


def _gpu_quantize(xd, rows, cols, ld, tag, gran, rnd, seed, offset, inv, want_q=True, want_t=True, bits=8):
    dt = {Q.INT8: torch.int8, Q.FP16: torch.float16, Q.FP32: torch.float32}[tag]
    q = empty((rows, cols), dt) if want_q else None
    qt = empty((cols, rows), dt) if want_t else None
    if q is not None:
        q.fill_(3)
    if qt is not None:
        qt.fill_(3)
    Q.qsync_quantize(xd, rows, cols, ld, tag, bits, GRAN[gran], RND[rnd], seed, offset, inv, q, qt)
    return q, qt


QSHAPES = [(16, 16), (16, 8), (48, 24), (128, 128), (256, 136), (144, 1000), (1024, 768), (5, 7), (17, 40), (24, 16),
           (130, 66), (2048, 64)]


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("gran", ["tensor", "row", "col"])
@pytest.mark.parametrize("rnd", ["nearest", "stochastic", "floor"])
def test_quantize_int8(dtype, gran, rnd):
    rng = np.random.default_rng(3)
    for rows, cols in QSHAPES:
        say("quantize", dtype.__name__, gran, rnd, rows, cols)
        x = _data(rng, (rows, cols), dtype, 0.7)
        x[0, 0] = 0
        seed, offset = 0x1234_5678_9ABC_DEF0 + rows, (1 << 64) - 5 if rows == 48 else 1000 * cols
        amax = orc.absmax(x, gran)
        so, io = orc.scales_from_amax(amax)
        want = orc.quantize_int(x, io, gran, rnd, seed, offset)
        q, qt = _gpu_quantize(dev(x), rows, cols, cols, Q.INT8, gran, rnd, seed, offset, dev(io))
        assert_bits_equal(host(q), want, "codes")
        assert_bits_equal(host(qt), want.T, "transposed codes")
    # only one of the two outputs; fewer bits
    x = _data(rng, (64, 64), dtype)
    so, io = orc.scales_from_amax(orc.absmax(x, gran), 5)
    want = orc.quantize_int(x, io, gran, rnd, 9, 9, bits=5)
    q, _ = _gpu_quantize(dev(x), 64, 64, 64, Q.INT8, gran, rnd, 9, 9, dev(io), True, False, bits=5)
    _, qt = _gpu_quantize(dev(x), 64, 64, 64, Q.INT8, gran, rnd, 9, 9, dev(io), False, True, bits=5)
    assert_bits_equal(host(q), want, "codes 5 bit")
    assert_bits_equal(host(qt), want.T, "transposed codes 5 bit")
    assert np.abs(want).max() == 15


def test_quantize_strided_input_and_special_values():
    rng = np.random.default_rng(4)
    for ld in (300, 304):                                      # ld 300: rows not 16-byte multiples -> scalar path
        big = _data(rng, (96, ld), np.float16)
        x = big[:, 8:8 + 256]
        so, io = orc.scales_from_amax(orc.absmax(x))
        say("quantize strided", ld)
        q, qt = _gpu_quantize(dev(big)[:, 8:264], 96, 256, ld, Q.INT8, "tensor", "stochastic", 5, 0, dev(io))
        want = orc.quantize_int(np.ascontiguousarray(x), io, "tensor", "stochastic", 5, 0)
        assert_bits_equal(host(q), want, "strided codes")
        assert_bits_equal(host(qt), want.T, "strided transposed codes")
    # ties, +-amax, subnormal inputs, exact integers
    say("quantize special values")
    t = np.zeros((16, 16), np.float32)
    t[0, :8] = [127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5]
    t[1, :4] = [-127.0, 1e-41, -1e-41, 126.5]
    so, io = orc.scales_from_amax(orc.absmax(t))
    for rnd in ("nearest", "stochastic", "floor"):
        q, qt = _gpu_quantize(dev(t), 16, 16, 16, Q.INT8, "tensor", rnd, 11, 3, dev(io))
        assert_bits_equal(host(q), orc.quantize_int(t, io, "tensor", rnd, 11, 3), f"special {rnd}")
    assert host(q).min() >= -127


@pytest.mark.parametrize("src", [np.float32, np.float16])
@pytest.mark.parametrize("tag", [Q.FP16, Q.FP32])
def test_cast_and_transpose(src, tag):
    rng = np.random.default_rng(5)
    for rows, cols in [(1, 1), (64, 64), (70, 130), (300, 96), (33, 1000), (256, 200), (72, 1032), (8, 8), (4096, 64),
                       (520, 8)]:
        say("cast", src.__name__, tag, rows, cols)
        x = _data(rng, (rows, cols), src, 100.0)
        x[0, 0] = 1.0 + 2.0**-11 if src == np.float32 else x[0, 0]     # an exact tie for binary16
        q, qt = _gpu_quantize(dev(x), rows, cols, cols, tag, "tensor", "nearest", 0, 0, None)
        want = orc.cast_fp16(x) if tag == Q.FP16 else x.astype(np.float32)
        assert_bits_equal(host(q), want, "cast")
        assert_bits_equal(host(qt), want.T, "cast transposed")
        q1, _ = _gpu_quantize(dev(x), rows, cols, cols, tag, "tensor", "nearest", 0, 0, None, True, False)
        _, qt1 = _gpu_quantize(dev(x), rows, cols, cols, tag, "tensor", "nearest", 0, 0, None, False, True)
        assert_bits_equal(host(q1), want, "cast, plain copy alone")
        assert_bits_equal(host(qt1), want.T, "cast, transposed copy alone")


@pytest.mark.parametrize("adt", [np.int32, np.int8])
@pytest.mark.parametrize("ydt", [np.float32, np.float16])
def test_dequantize(adt, ydt):
    rng = np.random.default_rng(6)
    for rows, cols in [(1, 1), (64, 64), (37, 53), (256, 1024), (100, 12)]:
        say("dequantize", adt.__name__, ydt.__name__, rows, cols)
        lim = 127 if adt == np.int8 else 2_000_000
        a = rng.integers(-lim, lim + 1, size=(rows, cols)).astype(adt)
        rs = rng.uniform(0.5, 2, rows).astype(np.float32)
        cs = rng.uniform(1e-4, 2e-4, cols).astype(np.float32)
        cb = rng.standard_normal(cols).astype(np.float32)
        for use in [(False, False, False), (True, False, False), (False, True, True), (True, True, True)]:
            y = empty((rows, cols), TORCH[ydt])
            Q.qsync_dequantize(dev(a), rows, cols, cols, dev(rs) if use[0] else None, dev(cs) if use[1] else None,
                               0.01, dev(cb) if use[2] else None, y)
            want = orc.dequantize(a, 0.01, rs if use[0] else None, cs if use[1] else None, cb if use[2] else None,
                                  np.float64)
            assert_close(host(y), want, "dequantize")
    # strided input
    a = rng.integers(-1000, 1000, size=(20, 64)).astype(adt if adt == np.int32 else np.int8)
    y = empty((20, 40), TORCH[ydt])
    Q.qsync_dequantize(dev(a)[:, 4:44], 20, 40, 64, None, None, 0.5, None, y)
    assert_close(host(y), a[:, 4:44] * 0.5, "dequantize strided")


def test_dequantize_to_binary16_rounds_the_exact_product_once():
    """int8 codes times one binary32 scale, binary16 output: the result is the exact product rounded once, bit
    for bit, also on inputs where rounding to binary32 first would give the other neighbour."""
    rng = np.random.default_rng(3)
    n = 1 << 18
    scales = (rng.uniform(0.5, 1.0, size=n).astype(np.float32) * np.float32(2.0 ** -7))
    codes = rng.integers(-127, 128, size=n).astype(np.int8)
    twice = (codes.astype(np.float32) * scales).astype(np.float16)
    want = orc.dequantize(codes.reshape(-1, 1), 1.0, row_scale=scales, out_dtype=np.float16)
    assert (want.reshape(-1).view(np.uint16) != twice.view(np.uint16)).sum() >= 3
    say("dequantize once-rounded, per-row scales")
    y = empty((n, 1), torch.float16)
    Q.qsync_dequantize(dev(codes.reshape(-1, 1)), n, 1, 1, dev(scales), None, 1.0, None, y)
    assert_bits_equal(host(y), want, "per-row scale")
    # the same pairs with the scale along the columns (the vector kernel), and a tensor scale held on the device
    rows = 64
    a = np.tile(codes[:4096].reshape(1, -1), (rows, 1))
    want = orc.dequantize(a, 1.0, col_scale=scales[:4096], out_dtype=np.float16)
    y = empty((rows, 4096), torch.float16)
    Q.qsync_dequantize(dev(a), rows, 4096, 4096, None, dev(scales[:4096]), 1.0, None, y)
    assert_bits_equal(host(y), want, "per-column scale")
    for i in np.flatnonzero(want[0].view(np.uint16) != twice[:4096].view(np.uint16))[:3]:
        a1 = rng.integers(-127, 128, size=(48, 272)).astype(np.int8)
        a1[0, 0] = codes[i]
        y = empty(a1.shape, torch.float16)
        Q.qsync_dequantize(dev(a1), 48, 272, 272, None, None, 1.0, None, y, tensor_scale_dev_opt=dev(scales[i:i + 1]))
        assert_bits_equal(host(y), orc.dequantize(a1, float(scales[i]), out_dtype=np.float16), "tensor scale on the device")


def test_empty_tensors_are_noops():
    s = empty(1, torch.float32)
    a = empty(1, torch.int32)
    Q.qsync_absmax_scale(s, 0, 16, 16, Q.PER_TENSOR, 8, s, s, None, None, None)
    Q.qsync_quantize(s, 0, 16, 16, Q.INT8, 8, 0, 0, 0, 0, s, s, None)
    Q.qsync_dequantize(a, 16, 0, 0, None, None, 1.0, None, s)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("rnd", ["nearest", "stochastic", "floor"])
def test_absmax_quantize_in_one_launch(dtype, rnd):
    """qsync_absmax_quantize: maximum, scales, codes and transposed codes equal the oracle's absmax ->
    scales_from_amax -> quantize_int bit for bit -- on shapes the single launch serves (one to 128 workgroups, ragged
    patch tails), on shapes it hands to the two launches (odd columns, large tensors), with the
    wait for the other workgroups cut to zero polls (every workgroup but the last then finds the maximum by itself),
    and on repeated calls that share one workspace without clearing it."""
    rng = np.random.default_rng(31)
    shapes = [(64, 128), (272, 1000), (1008, 72), (4096, 768), (2048, 2048), (48, 8200), (130, 72), (3, 5), (257, 1001)]
    w = ws(max(Q.qsync_absmax_quantize_workspace_bytes(r, c) for r, c in shapes))       # zero-filled once
    for rows, cols in shapes:
        x = _data(rng, (rows, cols), dtype, sigma=0.3)
        x[rows // 2, cols // 3] = dtype(-7.5)                                          # the maximum, negative
        xd = dev(x)
        amax = orc.absmax(x, "tensor")
        so, io = orc.scales_from_amax(amax)
        want = orc.quantize_int(x, io, "tensor", rnd, 77, 1234)
        for polls in (-1, 0, 3):
            for with_t in (True, False):
                if with_t and rows % 16 != 0:
                    continue
                say("absmax_quantize", dtype.__name__, rnd, rows, cols, "polls", polls, "transposed", with_t)
                s, iv, am = empty(1, torch.float32), empty(1, torch.float32), empty(1, torch.float32)
                q = torch.full((rows, cols), 99, dtype=torch.int8, device="cuda")
                qT = torch.full((cols, rows), 99, dtype=torch.int8, device="cuda") if with_t else None
                Q.qsync_absmax_quantize(xd, rows, cols, 8, RND[rnd], 77, 1234, s, iv, am, q, qT, w, polls)
                torch.cuda.synchronize()
                assert_bits_equal(host(am), amax, "amax")
                assert_bits_equal(host(s), so, "scale")
                assert_bits_equal(host(iv), io, "inverse scale")
                assert_bits_equal(host(q), want, "codes")
                if with_t:
                    assert_bits_equal(host(qT), want.T, "transposed codes")
    # the workspace's ticket word is back at zero: the separate maximum pass can use the same buffer next
    assert int(w[:4].view(torch.int32).item()) == 0
    x = _data(rng, (512, 4096), dtype)
    s, iv, am = empty(1, torch.float32), empty(1, torch.float32), empty(1, torch.float32)
    Q.qsync_absmax_scale(dev(x), 512, 4096, 4096, Q.PER_TENSOR, 8, s, iv, am, None, w)
    torch.cuda.synchronize()
    assert_bits_equal(host(am), orc.absmax(x, "tensor"), "amax by the separate pass on the shared workspace")


def test_absmax_quantize_all_zero_and_lower_bits():
    w = ws(Q.qsync_absmax_quantize_workspace_bytes(128, 256))
    z = torch.zeros(64, 128, dtype=torch.float16, device="cuda")
    s, iv, am = empty(1, torch.float32), empty(1, torch.float32), empty(1, torch.float32)
    q = torch.full((64, 128), 99, dtype=torch.int8, device="cuda")
    Q.qsync_absmax_quantize(z, 64, 128, 8, Q.ROUND_NEAREST, 0, 0, s, iv, am, q, None, w)
    torch.cuda.synchronize()
    assert s.item() == 1.0 and iv.item() == 1.0 and am.item() == 0.0 and int(q.abs().max().item()) == 0
    rng = np.random.default_rng(8)
    x = _data(rng, (128, 256), np.float32)
    so, io = orc.scales_from_amax(orc.absmax(x, "tensor"), 5)
    want = orc.quantize_int(x, io, "tensor", "stochastic", 9, 9, bits=5)
    q = torch.empty(128, 256, dtype=torch.int8, device="cuda")
    qT = torch.empty(256, 128, dtype=torch.int8, device="cuda")
    Q.qsync_absmax_quantize(dev(x), 128, 256, 5, Q.ROUND_STOCHASTIC, 9, 9, s, iv, am, q, qT, w)
    torch.cuda.synchronize()
    assert_bits_equal(host(s), so, "scale, 5 bits")
    assert_bits_equal(host(q), want, "codes, 5 bits")
    assert_bits_equal(host(qT), want.T, "transposed codes, 5 bits")
