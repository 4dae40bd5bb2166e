"""Pins for the oracle's absmax / scale / quantize / dequantize (CPU only).

What fixes the expected values: exact rational re-derivation (tests/bigint_ref.py), the
half-step error bound of nearest rounding, E[UQ(x)] = x and Var = q^2 D / 6 for stochastic
rounding (paper: Indicator section and Prop. 2), and the code range of a symmetric b-bit code.
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import qsync_oracle as orc
from tests import bigint_ref as ref

F = lambda v: Fraction(float(v))


def _brute_quantize(x, gran, mode, seed=0, offset=0, bits=8):
    rows, cols = x.shape
    absx = [[abs(F(x[r, c])) for c in range(cols)] for r in range(rows)]
    if gran == "tensor":
        am = [max(max(row) for row in absx)]
    elif gran == "row":
        am = [max(row) for row in absx]
    else:
        am = [max(absx[r][c] for r in range(rows)) for c in range(cols)]
    pairs = [ref.scale_pair(a, bits) for a in am]
    pick = lambda r, c: pairs[0] if gran == "tensor" else (pairs[r] if gran == "row" else pairs[c])
    codes = [[ref.quantize_scalar(F(x[r, c]), pick(r, c)[1], mode,
                                  ref.draw16(seed, offset, r * cols + c), bits)
              for c in range(cols)] for r in range(rows)]
    return am, pairs, codes


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("gran", ["tensor", "row", "col"])
@pytest.mark.parametrize("mode", ["nearest", "stochastic", "floor"])
def test_quantize_matches_rational_bruteforce(dtype, gran, mode):
    rng = np.random.default_rng(hash((str(dtype), gran, mode)) % 2**32)
    for shape, sigma in [((5, 7), 1.0), ((8, 8), 1e-3), ((3, 17), 40.0)]:
        x = (rng.standard_normal(shape) * sigma).astype(dtype)
        x[0, 0] = 0
        am, pairs, codes = _brute_quantize(x, gran, mode, seed=77, offset=2**33 + 1)
        amax = orc.absmax(x, gran)
        s, inv = orc.scales_from_amax(amax)
        assert [F(a) for a in amax] == am
        assert [F(v) for v in s] == [p[0] for p in pairs]
        assert [F(v) for v in inv] == [p[1] for p in pairs]
        got = orc.quantize_int(x, inv, gran, mode, seed=77, offset=2**33 + 1)
        assert got.dtype == np.int8
        assert got.tolist() == codes


def test_hand_built_cases():
    # all-zero tensor: scale 1, codes 0
    z = np.zeros((3, 4), np.float32)
    s, inv = orc.scales_from_amax(orc.absmax(z))
    assert s[0] == 1 and inv[0] == 1
    assert not orc.quantize_int(z, inv).any()
    assert not orc.quantize_int(z, inv, rounding="stochastic", seed=3).any()
    # single non-zero and +-amax elements map to +-127
    x = np.zeros((2, 5), np.float32); x[1, 2] = -3.25; x[0, 4] = 3.25
    s, inv = orc.scales_from_amax(orc.absmax(x))
    q = orc.quantize_int(x, inv)
    assert q[1, 2] == -127 and q[0, 4] == 127 and np.count_nonzero(q) == 2
    for seed in range(50):          # stochastic rounding of an exact integer never moves it
        qs = orc.quantize_int(x, inv, rounding="stochastic", seed=seed)
        assert qs[1, 2] == -127 and qs[0, 4] == 127
    # exact ties go to the even code: amax 127 gives inverse scale exactly 1
    t = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5]], np.float32)
    s, inv = orc.scales_from_amax(orc.absmax(t))
    assert inv[0] == 1.0
    assert orc.quantize_int(t, inv).tolist() == [[127, 0, 2, 2, 0, -2, -2, 4]]
    assert orc.quantize_int(t, inv, rounding="floor").tolist() == [[127, 0, 1, 2, -1, -2, -3, 3]]
    # negative values under stochastic rounding move between floor and floor+1 (not towards zero)
    n = np.array([[127.0, -2.25]], np.float32)
    seen = {int(orc.quantize_int(n, inv, rounding="stochastic", seed=sd)[0, 1]) for sd in range(200)}
    assert seen == {-3, -2}
    # fewer bits: qmax = 2^(b-1) - 1
    for bits in (2, 4, 7):
        s, inv = orc.scales_from_amax(orc.absmax(x), bits)
        q = orc.quantize_int(x, inv, bits=bits)
        assert q.max() == orc.qmax_of(bits) and q.min() == -orc.qmax_of(bits)
    with pytest.raises(ValueError):
        orc.qmax_of(9)


@pytest.mark.parametrize("gran", ["tensor", "row", "col"])
def test_nearest_error_at_most_half_a_step(gran):
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((64, 96)) * rng.uniform(0.01, 30, size=(64, 1))).astype(np.float32)
    amax = orc.absmax(x, gran)
    s, inv = orc.scales_from_amax(amax)
    q = orc.quantize_int(x, inv, gran, "nearest")
    sb = s.reshape({"tensor": (1, 1), "row": (-1, 1), "col": (1, -1)}[gran]).astype(np.float64)
    err = np.abs(x.astype(np.float64) - q.astype(np.float64) * sb)
    # half a step, plus the rounding of the inverse scale and of the product (a few 2^-24 of |x|)
    assert np.all(err <= 0.5 * sb * (1 + 2e-6) + 4 * 2.0**-24 * np.abs(x))
    assert q.min() >= -127 and q.max() <= 127
    # the dequantizer is the code times the scale
    xh = orc.dequantize(q, 1.0, row_scale=s if gran == "row" else None, col_scale=s if gran == "col" else None) \
        if gran != "tensor" else orc.dequantize(q, float(s[0]))
    np.testing.assert_allclose(xh, q * sb, rtol=1e-7)


def test_dequantize_with_row_and_column_scale_and_bias_exact_rational():
    """x_hat = code * q_tensor * q_row * q_col + bias on exact rationals, rounded once to the output type
    (Indicator section: the dequantized scalar; Cost Mapper paragraph: layer-wise and channel-wise dequantizers)."""
    from fractions import Fraction
    rng = np.random.default_rng(77)
    for dtype, lo, hi in ((np.int8, -127, 128), (np.int32, -(1 << 16), 1 << 16)):
        a = rng.integers(lo, hi, size=(5, 7)).astype(dtype)
        rs = rng.uniform(1e-3, 1.0, size=5).astype(np.float32)
        cs = rng.uniform(1e-3, 1.0, size=7).astype(np.float32)
        cb = rng.standard_normal(7).astype(np.float32)
        ts = np.float32(0.37)
        for use_r, use_c, use_b in [(True, True, True), (True, False, True), (False, True, False), (True, True, False),
                                    (False, False, True)]:
            for out, rnd in ((np.float32, ref.round_f32), (np.float16, ref.round_f16)):
                got = orc.dequantize(a, float(ts), rs if use_r else None, cs if use_c else None, cb if use_b else None, out)
                assert got.dtype == out
                for r in range(5):
                    for c in range(7):
                        v = Fraction(int(a[r, c])) * Fraction(float(ts))
                        if use_r: v *= Fraction(float(rs[r]))
                        if use_c: v *= Fraction(float(cs[c]))
                        if use_b: v += Fraction(float(cb[c]))
                        assert Fraction(float(got[r, c])) == rnd(v), (dtype, use_r, use_c, use_b, out, r, c)


def test_dequantized_binary16_operand_is_rounded_once():
    """The binary16 operand of the FP16 backward is the exact product code * scale rounded once.  Rounding the
    product to binary32 first and narrowing afterwards differs on some inputs; the search below finds such
    inputs (so the test bites) and the oracle must return the once-rounded value on them."""
    from fractions import Fraction
    rng = np.random.default_rng(3)
    scales = rng.uniform(0.5, 1.0, size=200000).astype(np.float32) * np.float32(2.0 ** -7)
    codes = rng.integers(3, 128, size=scales.size).astype(np.int8)
    once = (codes.astype(np.float64) * scales.astype(np.float64)).astype(np.float16)          # exact in double
    twice = (codes.astype(np.float32) * scales).astype(np.float16)
    hard = np.flatnonzero(once.view(np.uint16) != twice.view(np.uint16))
    assert hard.size >= 3, "no input separates one rounding from two"
    for i in hard[:20]:
        exact = Fraction(int(codes[i])) * Fraction(float(scales[i]))
        want = ref.round_f16(exact)
        assert Fraction(float(once[i])) == want and Fraction(float(twice[i])) != want
        got = orc.dequantize(codes[i:i + 1].reshape(1, 1), float(scales[i]), out_dtype=np.float16)
        assert Fraction(float(got[0, 0])) == want
        out = orc.fp16_backward_of_int8_forward(codes[i:i + 1].reshape(1, 1), scales[i:i + 1], codes[i:i + 1].reshape(1, 1),
                                                scales[i:i + 1], "row", np.zeros((1, 1), np.float32))
        assert Fraction(float(out["xh"][0, 0])) == want and Fraction(float(out["wh"][0, 0])) == want


def test_codes_never_reach_minus_128():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((257, 33)).astype(np.float32)
    x[3, 3] = -x.__abs__().max() * 1.0000001        # most negative element defines amax
    _, inv = orc.scales_from_amax(orc.absmax(x))
    for mode in ("nearest", "stochastic", "floor"):
        q = orc.quantize_int(x, inv, rounding=mode, seed=1)
        assert q.min() >= -127 and q.max() <= 127


def test_stochastic_rounding_unbiased_and_variance():
    """E[UQ(x)] = x and per-element variance q^2 f(1-f); summed over uniform residuals q^2 D/6 (Prop. 2)."""
    rng = np.random.default_rng(8)
    D = 512
    x = rng.uniform(-1, 1, size=(1, D)).astype(np.float32)
    x[0, 0] = 1.0
    s, inv = orc.scales_from_amax(orc.absmax(x))
    nseeds = 4096
    acc = np.zeros(D); acc2 = np.zeros(D)
    for seed in range(nseeds):
        c = orc.quantize_int(x, inv, rounding="stochastic", seed=seed, offset=seed * 64).astype(np.float64)[0]
        acc += c; acc2 += c * c
    mean = acc / nseeds
    var = acc2 / nseeds - mean**2
    v = (x * inv).astype(np.float32).astype(np.float64)[0]
    f = v - np.floor(v)
    sigma = np.sqrt(np.maximum(f * (1 - f), 1e-12) / nseeds)
    assert np.all(np.abs(mean - v) <= 4.5 * sigma + 2.0**-15)
    np.testing.assert_allclose(var.sum(), (f * (1 - f)).sum(), rtol=0.02)
    # residuals uniform on (0,1): total variance of the codes ~ D/6, of the dequantized tensor q^2 D/6
    assert abs(var.sum() / (D / 6) - 1) < 0.1
    xhat_var = var * float(s[0])**2                     # Var[x_hat] = q^2 Var[code]
    assert abs(xhat_var.sum() / (float(s[0])**2 * D / 6) - 1) < 0.1


def test_fp16_cast_is_ieee_nearest_even():
    # spacing of binary16 in [1,2) is 2^-10: halfway points go to the even neighbour
    base = np.float32(1.0)
    ulp = np.float32(2.0**-10)
    x = np.array([base + ulp / 2, base + 3 * ulp / 2, base + ulp * np.float32(0.501), 65504.0, 65520.0, 2.0**-25, 2.0**-24 * 1.5],
                 np.float32)
    h = orc.cast_fp16(x)
    assert h[0] == np.float16(1.0) and h[1] == np.float16(1.0 + 2 * 2.0**-10) and h[2] == np.float16(1.0 + 2.0**-10)
    assert h[3] == np.float16(65504.0) and np.isinf(h[4])
    assert h[5] == 0 and h[6] == np.float16(2.0**-23)


def test_quantizing_the_patch_matrix_equals_expanding_the_quantized_activation():
    """A 3x3 im2col only copies activation values and inserts zeros, every activation value appears in it,
    and zero quantizes to zero: with a per-tensor scale the codes of the patch matrix are the patches of
    the codes.  This is what lets the GPU path quantize the NHWC activation once and expand int8 codes."""
    from paper_2407_02327_amd import workloads as wl
    rng = np.random.default_rng(40)
    act = np.abs(rng.standard_normal((2, 7, 5, 16))).astype(np.float16)
    x = wl.im2col_nhwc_3x3(act)
    a_act, a_x = orc.absmax(act.reshape(-1, 16), "tensor"), orc.absmax(x, "tensor")
    assert a_act.tobytes() == a_x.tobytes()
    _, inv = orc.scales_from_amax(a_x)
    q_of_patches = orc.quantize_int(x, inv, "tensor", "nearest")
    patches_of_q = wl.im2col_nhwc_3x3(orc.quantize_int(act.reshape(-1, 16), inv, "tensor", "nearest").reshape(act.shape))
    assert np.array_equal(q_of_patches, patches_of_q)
    # hand check of one row: output pixel (n=1, h=0, w=4) is a corner: taps with h-1 or w+1 are zero
    m = (1 * 7 + 0) * 5 + 4
    row = patches_of_q[m].reshape(3, 3, 16)
    assert not row[0].any() and not row[:, 2].any()
    centre = orc.quantize_int(act[1, 0, 4].reshape(1, 16), inv, "tensor", "nearest")[0]
    assert np.array_equal(row[1, 1], centre)
