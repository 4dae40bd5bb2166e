"""CPU oracle for the quantized training operators (TEST INFRASTRUCTURE ONLY).

A plain, slow, obviously-correct numpy statement of what the hot path computes:
absmax -> scale -> INT8 quantize (nearest-even or seeded stochastic rounding) or
FP16 cast -> forward GEMM Y = X W^T -> backward GEMMs dX = dY W, dW = dY^T X ->
dequantize with scale and bias.  It is independent of the HIP library: it shares
no code, tables or helpers with it and must never be imported by the product
path.  Only the tests, the smoke check and the benchmark's CPU-baseline leg use it.

Where the paper fixes the arithmetic the function cites the passage; where the
paper is silent the docstring states the reading taken.

Pins (see tests/test_oracle_*.py): brute-force big-integer re-derivation on tiny
inputs, the <= scale/2 error bound of nearest rounding, unbiasedness and the
D/6 variance law of stochastic rounding (Prop. 2), code range, the forward
identity of the Prop. 2 proof (integer GEMM times scales == GEMM of dequantized
tensors), the published Philox4x32-10 known answers and rocRAND's host engine for the generator, and math.fsum
triple loops for the floating-point contractions; for the 3x3 convolution scipy's
2-D correlation, six-deep loops, single-tap shifts, a hand-worked example and the
adjoint identities.
Parity unpinned: nothing in this file.
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np

INT8, FP16, FP32 = 8, 16, 32

_F32 = np.float32
_MASK32 = np.uint64(0xFFFFFFFF)

# Philox4x32 multipliers and Weyl key increments (Salmon, Moraes, Dror, Shaw:
# "Parallel random numbers: as easy as 1, 2, 3", SC'11, Philox4x32 definition).
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = np.uint64(0x9E3779B9)
_PHILOX_W1 = np.uint64(0xBB67AE85)


# --------------------------------------------------------------------------- RNG
def philox4x32_10(counter: np.ndarray, key: Tuple[int, int]) -> np.ndarray:
    """Ten rounds of Philox4x32 on an array of 128-bit counters.

    counter: [..., 4] uint32 words, least significant first.  key: two 32-bit words.
    One round maps (c0,c1,c2,c3) to (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0));
    the key is advanced by the Weyl constants between rounds.
    """
    c = counter.astype(np.uint64)
    c0, c1, c2, c3 = c[..., 0], c[..., 1], c[..., 2], c[..., 3]
    k0, k1 = np.uint64(key[0] & 0xFFFFFFFF), np.uint64(key[1] & 0xFFFFFFFF)
    for _ in range(10):
        p0 = _PHILOX_M0 * c0
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
        k0 = (k0 + _PHILOX_W0) & _MASK32
        k1 = (k1 + _PHILOX_W1) & _MASK32
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def sr_draws(seed: int, offset: int, numel: int) -> np.ndarray:
    """The 16-bit uniform draw of every element 0..numel-1 of a tensor.

    Reading (the paper names no generator; stochastic rounding is only said to be
    driven by the residual, Indicator section): element i (row-major linear index)
    belongs to group g = i // 8; the group's Philox counter is the 128-bit integer
    offset + g, the key is (seed mod 2^32, seed >> 32); the four output words are
    cut into eight 16-bit draws, element i takes draw i mod 8, i.e. word (i mod 8)//2,
    low half first.
    """
    groups = (numel + 7) // 8
    g = np.arange(groups, dtype=np.uint64)
    lo = np.uint64(offset & 0xFFFFFFFFFFFFFFFF) + g          # wraps mod 2^64
    carry = (lo < g).astype(np.uint64) + np.uint64((offset >> 64) & 0xFFFFFFFF)
    ctr = np.stack([lo & _MASK32, lo >> np.uint64(32), carry & _MASK32,
                    np.zeros_like(lo)], axis=-1).astype(np.uint32)
    words = philox4x32_10(ctr, (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF))      # [groups, 4]
    halves = np.stack([words & np.uint32(0xFFFF), words >> np.uint32(16)], axis=-1)  # [groups, 4, 2]
    return halves.reshape(-1)[:numel].astype(np.uint16)


# ------------------------------------------------------------------ absmax, scale
def absmax(x: np.ndarray, gran: str = "tensor") -> np.ndarray:
    """max |x| of the tensor ("tensor"), of each row ("row") or each column ("col"), in fp32.

    The paper's min-max kernel returns the absolute tensor-wise value (Backend
    section, Minmax Optimization); fp16 inputs are widened exactly.
    """
    a = np.abs(x.astype(_F32))
    if a.size == 0:
        raise ValueError("absmax of an empty tensor is undefined")
    if gran == "tensor":
        return a.max().reshape(1)
    if gran == "row":
        return a.max(axis=1)
    if gran == "col":
        return a.max(axis=0)
    raise ValueError(gran)


def qmax_of(bits: int) -> int:
    if not 2 <= bits <= 8:
        raise ValueError("bits must be in 2..8")
    return (1 << (bits - 1)) - 1


def scales_from_amax(amax: np.ndarray, bits: int = 8) -> Tuple[np.ndarray, np.ndarray]:
    """Symmetric fixed-point scale q = amax/qmax and its inverse qmax/amax, each one fp32 division.

    Zero-point z = 0 (symmetric reading of x_bar = (x - z)/q, Indicator section).
    An all-zero tensor or row gets q = 1 and inverse 1 so that its codes are 0.
    """
    amax = amax.astype(_F32)
    q = _F32(qmax_of(bits))
    zero = amax == 0
    safe = np.where(zero, _F32(1), amax)
    s = np.where(zero, _F32(1), safe / q).astype(_F32)
    inv = np.where(zero, _F32(1), q / safe).astype(_F32)
    return s, inv


def _broadcast(vec: np.ndarray, gran: str, shape) -> np.ndarray:
    vec = np.asarray(vec, dtype=_F32)
    if gran == "tensor":
        return vec.reshape(1, 1)
    if gran == "row":
        return vec.reshape(shape[0], 1)
    if gran == "col":
        return vec.reshape(1, shape[1])
    raise ValueError(gran)


# ------------------------------------------------------------------------ quantize
def quantize_int(x: np.ndarray, inv_scale: np.ndarray, gran: str = "tensor", rounding: str = "nearest",
                 seed: int = 0, offset: int = 0, bits: int = 8) -> np.ndarray:
    """Fixed-point codes round(x / q), clamped to [-qmax, qmax], stored as int8.

    x_bar = x * (1/q) is one fp32 multiply (Indicator section: x_bar = (x - z)/q, z = 0).
    "nearest": ties to even.  "floor": round down (Discussion, Quantization by Floor).
    "stochastic": round up with probability floor(frac * 2^16) / 2^16, frac = x_bar - floor(x_bar),
    using the element's 16-bit draw u from `sr_draws`: up iff u < floor(frac * 2^16).
    This is the unbiased quantizer of the Indicator section (E[UQ(x)] = x) up to 2^-16 of a step.
    """
    qmax = _F32(qmax_of(bits))
    xf = x.astype(_F32)
    v = (xf * _broadcast(inv_scale, gran, x.shape)).astype(_F32)
    if rounding == "nearest":
        c = np.rint(v)
    elif rounding == "floor":
        c = np.floor(v)
    elif rounding == "stochastic":
        fl = np.floor(v)
        fr = (v - fl).astype(_F32)                       # exact: fl and v share a binade or fl is adjacent
        thr = (fr * _F32(65536.0)).astype(np.uint32)     # exact product, truncation
        u = sr_draws(seed, offset, x.size).reshape(x.shape).astype(np.uint32)
        c = fl + (u < thr).astype(_F32)
    else:
        raise ValueError(rounding)
    c = np.minimum(np.maximum(c, -qmax), qmax)
    return c.astype(np.int8)


def cast_fp16(x: np.ndarray) -> np.ndarray:
    """IEEE round-to-nearest-even narrowing to binary16 (the FP16 precision tag)."""
    return x.astype(np.float16)


def cast_fp16_stochastic(x: np.ndarray, seed: int = 0, offset: int = 0, k: int = 9) -> np.ndarray:
    """Floating-point stochastic quantization to binary16 (Appendix, Proposition 2, the two-case rule
    for the rounded value): with x = s 2^e (1 + m), the mantissa is truncated to k bits and the value moves
    up by eps = 2^-k (in units of 2^e) with probability (m - floor_k(m)) / eps.

    Worked out on the binary32 significand as integers.  sig * 2^(e-23) is |x| (sig carries the implicit
    one); D = (23 - k) + max(0, -14 - e) low bits are dropped, so that below the binary16 normal range
    the spacing stays that of the target format (2^(-14-k)); the dropped part rem gives the threshold
    floor(rem * 2^16 / 2^D) and the element's 16-bit draw u (same Philox mapping as the fixed-point
    quantizer) rounds up iff u < threshold.  The result is exactly representable in binary16 unless it
    reaches 2^16, which becomes infinity as in IEEE narrowing.  binary16 input is returned unchanged.
    The default k = 9 is the value the paper states for float16 (remark after Prop. 2 of the Indicator
    section); k = 10 keeps the full binary16 mantissa.
    """
    if x.dtype == np.float16:
        return x.copy()
    if not 7 <= k <= 10:
        raise ValueError("k must be 7..10")
    xf = np.ascontiguousarray(x, dtype=_F32)
    bits = xf.view(np.uint32).astype(np.uint64)
    neg = (bits >> np.uint64(31)) & np.uint64(1)
    eb = ((bits >> np.uint64(23)) & np.uint64(0xFF)).astype(np.int64)
    mant = bits & np.uint64(0x7FFFFF)
    sig = np.where(eb == 0, mant, mant | np.uint64(1 << 23)).astype(np.uint64)
    e = np.where(eb == 0, -126, eb - 127)
    D = (23 - k) + np.maximum(0, -14 - e)
    D = np.minimum(D, 40).astype(np.uint64)
    kept = sig >> D
    rem = sig & ((np.uint64(1) << D) - np.uint64(1))
    thr = np.where(D >= 16, rem >> np.maximum(D, np.uint64(16)) - np.uint64(16),
                   rem << (np.uint64(16) - np.minimum(D, np.uint64(16))))
    u = sr_draws(seed, offset, x.size).reshape(x.shape).astype(np.uint64)
    res = kept + (u < thr).astype(np.uint64)
    val = np.ldexp(res.astype(np.float64), (e - 23 + D.astype(np.int64)).astype(np.int64))
    val = np.where(neg == 1, -val, val)
    with np.errstate(over="ignore"):
        return val.astype(np.float16)


def dequantize(a: np.ndarray, tensor_scale: float = 1.0, row_scale: Optional[np.ndarray] = None,
               col_scale: Optional[np.ndarray] = None, col_bias: Optional[np.ndarray] = None,
               out_dtype=np.float32) -> np.ndarray:
    """x_hat = code * q (+ bias): the dequantizer of the Indicator section, per tensor, row or column.

    Scales are fp32 values; the product is formed in double and rounded once.
    """
    y = a.astype(np.float64) * float(_F32(tensor_scale))
    if row_scale is not None:
        y = y * np.asarray(row_scale, _F32).astype(np.float64).reshape(-1, 1)
    if col_scale is not None:
        y = y * np.asarray(col_scale, _F32).astype(np.float64).reshape(1, -1)
    if col_bias is not None:
        y = y + np.asarray(col_bias, _F32).astype(np.float64).reshape(1, -1)
    return y.astype(out_dtype)


# --------------------------------------------------------------------------- GEMMs
def int_gemm_nt(a_q: np.ndarray, b_q: np.ndarray) -> Tuple[np.ndarray, bool]:
    """acc[i,j] = sum_k a_q[i,k] * b_q[j,k] as int32 (two's-complement wrap) plus an overflow flag.

    The sum is formed by a float64 matrix product of the codes: every product is an
    integer of magnitude <= 2^14 and every partial sum stays below 2^53 for any
    contraction length < 2^39, so each floating-point addition is exact whatever the
    order and the result is the integer sum itself.  "Fixed-point calculation is done
    in INT32" (Backend section, Dequantization Fusion); the paper is silent on overflow,
    the reading here is wrap-around mod 2^32 with the event reported.
    """
    assert a_q.dtype == np.int8 and b_q.dtype == np.int8 and a_q.shape[1] == b_q.shape[1]
    assert a_q.shape[1] < (1 << 39)
    exact = a_q.astype(np.float64) @ b_q.astype(np.float64).T
    acc64 = exact.astype(np.int64)
    overflow = bool(acc64.size and (acc64.max() > 2**31 - 1 or acc64.min() < -2**31))
    acc32 = (acc64 & np.int64(0xFFFFFFFF)).astype(np.uint32).view(np.int32)
    return acc32, overflow


def float_gemm_nt(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """sum_k a[i,k] * b[j,k] in double over the given (already cast) operands."""
    return a.astype(np.float64) @ b.astype(np.float64).T


def naive_matmul_nt_f32(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Textbook triple loop in fp32, k innermost and sequential (small shapes only)."""
    m, k = a.shape
    n = b.shape[0]
    out = np.zeros((m, n), dtype=_F32)
    for i in range(m):
        for j in range(n):
            s = _F32(0)
            for t in range(k):
                s = _F32(s + _F32(a[i, t] * b[j, t]))
            out[i, j] = s
    return out


def qlinear_fwd(tag: int, xq: np.ndarray, sx, wq: np.ndarray, sw, bias: Optional[np.ndarray],
                out_dtype=np.float32):
    """Forward of one operator under precision tag INT8 / FP16 / FP32.

    INT8 (proof of Prop. 2, forward flow of a fixed-point kernel, zero-points 0):
    y = q_v q_w sum(v_q w_q) + b with q_w per tensor or per output channel; the dequantizer
    pairing follows the Cost Mapper paragraph (layer-wise input x channel-wise weight ->
    channel-wise dequantizer).  Returns (Y, int32 accumulators, overflow flag).
    FP16 / FP32: Y = X W^T + b over the cast / untouched operands, accumulated in double.
    Returns (Y, None, False).
    """
    if tag == INT8:
        acc, ovf = int_gemm_nt(xq, wq)
        sw = np.asarray(sw, _F32).reshape(-1)
        col = sw if sw.size > 1 else None
        ts = float(_F32(np.asarray(sx).reshape(-1)[0])) * (1.0 if col is not None else float(sw[0]))
        y = acc.astype(np.float64) * ts
        if col is not None:
            y = y * col.astype(np.float64).reshape(1, -1)
        if bias is not None:
            y = y + np.asarray(bias, _F32).astype(np.float64).reshape(1, -1)
        return y.astype(out_dtype), acc, ovf
    if tag in (FP16, FP32):
        want = np.float16 if tag == FP16 else np.float32
        assert xq.dtype == want and wq.dtype == want
        y = float_gemm_nt(xq, wq)
        if bias is not None:
            y = y + np.asarray(bias, _F32).astype(np.float64).reshape(1, -1)
        return y.astype(out_dtype), None, False
    raise ValueError(tag)


def qlinear_bwd(tag: int, dyq: np.ndarray, sdy, xq: np.ndarray, sx, wqb: np.ndarray, swb,
                dy_float: Optional[np.ndarray], dx_dtype=np.float16, dw_dtype=np.float32):
    """Backward of one operator: (dW, dX) = G[dY, C(v, x)] (Appendix, proof of Prop. 1).

    dX[m,k] = sum_n dY[m,n] W[n,k],  dW[n,k] = sum_m dY[m,n] X[m,k],  db[n] = sum_m dY[m,n].
    INT8 tag: both contractions run on codes with int32 accumulation.  dyq is the
    per-tensor quantized gradient; wqb holds codes of W [N,K] whose scale swb is per
    tensor or per column k (a scale along n would sit on the contraction axis and could
    not leave the integer sum); xq/sx are the forward's saved activation codes.
    dX = accX * sdy * swb[k], dW = accW * sdy * sx.  The paper itself runs this backward
    in FP16 (footnote in the Cost Mapper paragraph); that is what tag FP16 computes.
    db is a double sum of the unquantized gradient.  Defaults follow the paper's output
    types: dW fp32, dX fp16 (Backend section, Dequantization Fusion).
    Returns dict(dx, dw, db, acc_dx, acc_dw, overflow).
    """
    out = {"acc_dx": None, "acc_dw": None, "overflow": False, "db": None}
    if dy_float is not None:
        out["db"] = dy_float.astype(np.float64).sum(axis=0).astype(_F32)
    if tag == INT8:
        acc_dx, o1 = int_gemm_nt(dyq, np.ascontiguousarray(wqb.T))      # contraction over n
        acc_dw, o2 = int_gemm_nt(np.ascontiguousarray(dyq.T), np.ascontiguousarray(xq.T))  # over m
        sdy = float(_F32(np.asarray(sdy).reshape(-1)[0]))
        sxv = float(_F32(np.asarray(sx).reshape(-1)[0]))
        swb = np.asarray(swb, _F32).reshape(-1)
        dx = acc_dx.astype(np.float64) * sdy
        dx = dx * (swb.astype(np.float64).reshape(1, -1) if swb.size > 1 else float(swb[0]))
        dw = acc_dw.astype(np.float64) * (sdy * sxv)
        out.update(dx=dx.astype(dx_dtype), dw=dw.astype(dw_dtype), acc_dx=acc_dx, acc_dw=acc_dw,
                   overflow=o1 or o2)
        return out
    if tag in (FP16, FP32):
        dx = float_gemm_nt(dyq, np.ascontiguousarray(wqb.T))
        dw = float_gemm_nt(np.ascontiguousarray(dyq.T), np.ascontiguousarray(xq.T))
        out.update(dx=dx.astype(dx_dtype), dw=dw.astype(dw_dtype))
        return out
    raise ValueError(tag)


# ------------------------------------------------------- activation between operators
def gelu(x: np.ndarray) -> np.ndarray:
    """Exact GELU x * Phi(x) in double (erf form); used between the operators of the MLP chain."""
    xd = x.astype(np.float64)
    erf = np.vectorize(math.erf, otypes=[np.float64])
    return 0.5 * xd * (1.0 + erf(xd / math.sqrt(2.0)))


def gelu_grad(x: np.ndarray) -> np.ndarray:
    """d/dx [x Phi(x)] = Phi(x) + x phi(x) in double."""
    xd = x.astype(np.float64)
    erf = np.vectorize(math.erf, otypes=[np.float64])
    cdf = 0.5 * (1.0 + erf(xd / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * xd * xd) / math.sqrt(2.0 * math.pi)
    return cdf + xd * pdf


# ------------------------------------------------------------ indicator statistics
def effective_exponent(amax: float) -> int:
    """Exponent e of the largest magnitude, 2^e <= amax < 2^(e+1) (the "effective bits" the Indicator
    section derives from the data's magnitude); -126 for an all-zero tensor."""
    if not amax > 0:
        return -126
    return int(math.floor(math.log2(float(amax))))


def tensor_stats(x: np.ndarray) -> dict:
    """The per-tensor quantities the variance indicator needs (Indicator section, Prop. 3): squared
    Euclidean norm (double sum), absmax, effective exponent and dimensionality."""
    xd = x.astype(np.float64).reshape(-1)
    am = float(absmax(x, "tensor")[0]) if x.size else 0.0
    return dict(sumsq=float(np.dot(xd, xd)), amax=am, e=effective_exponent(am), D=int(x.size))


def variance_increment(kind: str, x: dict, v: dict, gv: dict, q_x: float = 0.0, q_v: float = 0.0,
                       eps: float = 2.0 ** -9, gamma: float = 1.0, d_o: int = 1, d_L: int = 1) -> dict:
    """Omega = gamma^2 d_o sigma_fp + (d_L - d_o) sigma_bp of one unary operator (Prop. 3 and the two
    case equations below it).  x, v, gv are tensor_stats of the parameter, the (dequantized) activation
    and the activation gradient; q_x, q_v the fixed-point scales; eps = 2^-k of the float format.
      fixed:  sigma_fp = (|x|^2 q_v^2 D_v + |v|^2 q_x^2 D_x) / 6
              sigma_bp = (|gv|^2 q_v^2 D_v + |v|^2 2^(2 e_gv) eps^2 D_gv) / 6
      float:  sigma_fp = eps^2 (|x|^2 2^(2 e_v) D_v + |v|^2 2^(2 e_x) D_x) / 6
              sigma_bp = eps^2 (|gv|^2 2^(2 e_v) D_v + |v|^2 2^(2 e_gv) D_gv) / 6
    """
    if kind == "fixed":
        s_fp = (x["sumsq"] * q_v ** 2 * v["D"] + v["sumsq"] * q_x ** 2 * x["D"]) / 6.0
        s_bp = (gv["sumsq"] * q_v ** 2 * v["D"] + v["sumsq"] * 4.0 ** gv["e"] * eps ** 2 * gv["D"]) / 6.0
    elif kind == "float":
        s_fp = eps ** 2 * (x["sumsq"] * 4.0 ** v["e"] * v["D"] + v["sumsq"] * 4.0 ** x["e"] * x["D"]) / 6.0
        s_bp = eps ** 2 * (gv["sumsq"] * 4.0 ** v["e"] * v["D"] + v["sumsq"] * 4.0 ** gv["e"] * gv["D"]) / 6.0
    else:
        raise ValueError(kind)
    return dict(sigma_fp=s_fp, sigma_bp=s_bp, omega=gamma ** 2 * d_o * s_fp + (d_L - d_o) * s_bp)


# ------------------------------------------------------------ whole-operator drivers
def fp16_backward_of_int8_forward(xq: np.ndarray, sx, wq: np.ndarray, sw, w_gran: str, dy: np.ndarray,
                                  dx_dtype=np.float16, dw_dtype=np.float32) -> dict:
    """Backward of a fixed-point operator the way the paper runs it (footnote in the Cost Mapper
    paragraph: the backward of fixed-point kernels is executed in FP16).

    The saved forward codes are dequantized and narrowed to binary16, the incoming gradient is narrowed
    to binary16, and the two contractions of the Prop. 1 proof run on those operands:
    dX = dY16 W16,  dW = dY16^T X16,  db = sum_m dY.

    The dequantized scalar of the Indicator section is x_hat = round(x_bar) * q_x, a product of an 8-bit
    code and a binary32 scale: at most 32 significant bits, so it is exact in double.  The binary16
    operand is that exact value rounded once to nearest even; no intermediate binary32 rounding is part
    of the definition.
    Returns dict(xh, wh, dyh, dx, dw, db).
    """
    sxv = float(_F32(np.asarray(sx).reshape(-1)[0]))
    xh = dequantize(xq, tensor_scale=sxv, out_dtype=np.float16)
    swv = np.asarray(sw, _F32).reshape(-1)
    if w_gran == "row":
        wh = dequantize(wq, row_scale=swv, out_dtype=np.float16)
    else:
        wh = dequantize(wq, tensor_scale=float(swv[0]), out_dtype=np.float16)
    dyh = cast_fp16(dy)
    b = qlinear_bwd(FP16, dyh, None, xh, None, wh, None, dy, dx_dtype, dw_dtype)
    return dict(xh=xh, wh=wh, dyh=dyh, dx=b["dx"], dw=b["dw"], db=b["db"])


def operator_fwd_bwd(tag: int, x: np.ndarray, w: np.ndarray, bias, dy: np.ndarray, w_gran: str = "row",
                     dy_round: str = "stochastic", seed: int = 0, offset: int = 0,
                     y_dtype=np.float32, dx_dtype=np.float16, dw_dtype=np.float32, bwd_tag: Optional[int] = None) -> dict:
    """absmax -> quantize/cast -> forward -> quantize dY -> backward, for one linear operator.

    Returns every intermediate (codes, scales, accumulators, outputs) so a test can
    compare each stage.  For INT8 with per-output-channel weights the backward uses a
    second quantization of W with one scale per input feature k (see qlinear_bwd).
    bwd_tag = FP16 with tag = INT8 selects the paper's own pairing: INT8 forward, FP16 backward
    on the dequantized saved codes (fp16_backward_of_int8_forward).
    """
    r = {}
    if tag == INT8 and bwd_tag == FP16:
        ax = absmax(x, "tensor"); sx, ix = scales_from_amax(ax)
        aw = absmax(w, w_gran); sw, iw = scales_from_amax(aw)
        xq = quantize_int(x, ix, "tensor", "nearest")
        wq = quantize_int(w, iw, w_gran, "nearest")
        y, acc, ovf = qlinear_fwd(INT8, xq, sx, wq, sw, bias, y_dtype)
        b = fp16_backward_of_int8_forward(xq, sx, wq, sw, w_gran, dy, dx_dtype, dw_dtype)
        r.update(sx=sx, sw=sw, xq=xq, wq=wq, y=y, acc=acc, overflow=ovf, **b)
        return r
    if tag == INT8:
        ax = absmax(x, "tensor"); sx, ix = scales_from_amax(ax)
        aw = absmax(w, w_gran); sw, iw = scales_from_amax(aw)
        xq = quantize_int(x, ix, "tensor", "nearest")
        wq = quantize_int(w, iw, w_gran, "nearest")
        y, acc, ovf = qlinear_fwd(INT8, xq, sx, wq, sw, bias, y_dtype)
        ady = absmax(dy, "tensor"); sdy, idy = scales_from_amax(ady)
        dyq = quantize_int(dy, idy, "tensor", dy_round, seed, offset)
        if w_gran == "row":
            awb = absmax(w, "col"); swb, iwb = scales_from_amax(awb)
            wqb = quantize_int(w, iwb, "col", "nearest")
        else:
            swb, wqb = sw, wq
        b = qlinear_bwd(INT8, dyq, sdy, xq, sx, wqb, swb, dy, dx_dtype, dw_dtype)
        r.update(sx=sx, sw=sw, xq=xq, wq=wq, y=y, acc=acc, sdy=sdy, dyq=dyq, swb=swb, wqb=wqb,
                 overflow=ovf or b["overflow"], **{k: b[k] for k in ("dx", "dw", "db", "acc_dx", "acc_dw")})
        return r
    if tag == FP16:
        xh, wh, dyh = cast_fp16(x), cast_fp16(w), cast_fp16(dy)
    elif tag == FP32:
        xh, wh, dyh = x.astype(_F32), w.astype(_F32), dy.astype(_F32)
    else:
        raise ValueError(tag)
    y, _, _ = qlinear_fwd(tag, xh, None, wh, None, bias, y_dtype)
    b = qlinear_bwd(tag, dyh, None, xh, None, wh, None, dy, dx_dtype, dw_dtype)
    r.update(xq=xh, wq=wh, dyq=dyh, y=y, overflow=False, **{k: b[k] for k in ("dx", "dw", "db")})
    return r


# ------------------------------------------------ 3x3 convolution (NHWC, stride 1, pad 1)
# The paper's convolution models run NHWC low-precision kernels (Experiment setup: "only the
# NHWC format is supported" below 16 bit); its forward/backward flow is the linear operator's
# (Appendix, proofs of Prop. 1 and Prop. 2) with the contraction running over the 3x3 window and
# the input channels.  The functions below are the definition written out tap by tap:
#   Y[b,h,w,n]  = sum_{kh,kw,c} X[b, h+kh-1, w+kw-1, c] * W[n,kh,kw,c]        (zero outside the image)
#   dX[b,h,w,c] = sum_{kh,kw,n} dY[b, h-(kh-1), w-(kw-1), n] * W[n,kh,kw,c]
#   dW[n,kh,kw,c] = sum_{b,h,w} dY[b,h,w,n] * X[b, h+kh-1, w+kw-1, c]
def _pad_hw(a: np.ndarray) -> np.ndarray:
    b, h, w, c = a.shape
    p = np.zeros((b, h + 2, w + 2, c), dtype=np.float64)
    p[:, 1:h + 1, 1:w + 1, :] = a
    return p


def conv3x3_fwd_f64(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """x [B,H,W,C], w [N,3,3,C] -> [B,H,W,N] in double (exact for integer codes: every partial sum < 2^53)."""
    b, h, wd, c = x.shape
    assert w.shape[1:] == (3, 3, c)
    xp, wf = _pad_hw(x), w.astype(np.float64)
    y = np.zeros((b, h, wd, w.shape[0]), dtype=np.float64)
    for kh in range(3):
        for kw in range(3):
            y += xp[:, kh:kh + h, kw:kw + wd, :] @ wf[:, kh, kw, :].T
    return y


def conv3x3_dgrad_f64(dy: np.ndarray, w: np.ndarray) -> np.ndarray:
    """dy [B,H,W,N], w [N,3,3,C] -> dX [B,H,W,C]: every output pixel scatters its gradient over its window."""
    b, h, wd, n = dy.shape
    assert w.shape[0] == n and w.shape[1:3] == (3, 3)
    c = w.shape[3]
    dxp = np.zeros((b, h + 2, wd + 2, c), dtype=np.float64)
    dyf, wf = dy.astype(np.float64), w.astype(np.float64)
    for kh in range(3):
        for kw in range(3):
            dxp[:, kh:kh + h, kw:kw + wd, :] += dyf @ wf[:, kh, kw, :]
    return dxp[:, 1:h + 1, 1:wd + 1, :]


def conv3x3_wgrad_f64(dy: np.ndarray, x: np.ndarray) -> np.ndarray:
    """dy [B,H,W,N], x [B,H,W,C] -> dW [N,3,3,C]."""
    b, h, wd, n = dy.shape
    c = x.shape[3]
    xp = _pad_hw(x)
    dyf = dy.astype(np.float64).reshape(-1, n)
    dw = np.zeros((n, 3, 3, c), dtype=np.float64)
    for kh in range(3):
        for kw in range(3):
            dw[:, kh, kw, :] = dyf.T @ xp[:, kh:kh + h, kw:kw + wd, :].reshape(-1, c)
    return dw


def _wrap_i32(exact: np.ndarray) -> Tuple[np.ndarray, bool]:
    acc64 = exact.astype(np.int64)
    ovf = bool(acc64.size and (acc64.max() > 2**31 - 1 or acc64.min() < -2**31))
    return (acc64 & np.int64(0xFFFFFFFF)).astype(np.uint32).view(np.int32), ovf


def conv3x3_operator_fwd_bwd(tag: int, act: np.ndarray, w: np.ndarray, bias, dy: np.ndarray, w_gran: str = "row",
                             dy_round: str = "stochastic", seed: int = 0, offset: int = 0,
                             y_dtype=np.float32, dx_dtype=np.float16, dw_dtype=np.float32) -> dict:
    """absmax -> quantize/cast -> forward -> quantize dY -> dgrad, wgrad for one 3x3 convolution.

    act [B,H,W,C]; w [N, 9*C] with k = (kh, kw, c); dy [B*H*W, N] (or [B,H,W,N]); outputs Y [B*H*W, N],
    dX [B*H*W, C], dW [N, 9*C].  The quantizers are the linear operator's (operator_fwd_bwd): activation
    and gradient per tensor, weights per tensor or per output channel ("row").  Reading for the data
    gradient with per-output-channel weights: the output channel n sits on dgrad's contraction axis, so
    dgrad uses a second quantization of W with one scale per input channel c (absmax over n, kh, kw) -- the
    convolution's counterpart of the per-input-feature scales of the linear backward (see qlinear_bwd).
    """
    b, h, wd, c = act.shape
    n = w.shape[0]
    assert w.shape == (n, 9 * c)
    m = b * h * wd
    dy2 = dy.reshape(m, n)
    r = {}
    if tag == INT8:
        ax = absmax(act.reshape(m, c), "tensor"); sx, ix = scales_from_amax(ax)
        aw = absmax(w, w_gran); sw, iw = scales_from_amax(aw)
        xq = quantize_int(act.reshape(m, c), ix, "tensor", "nearest")
        wq = quantize_int(w, iw, w_gran, "nearest")
        acc, o0 = _wrap_i32(conv3x3_fwd_f64(xq.reshape(b, h, wd, c), wq.reshape(n, 3, 3, c)).reshape(m, n))
        swv = np.asarray(sw, _F32).reshape(-1)
        sxv = float(_F32(np.asarray(sx).reshape(-1)[0]))
        y = acc.astype(np.float64) * (sxv if swv.size > 1 else sxv * float(swv[0]))
        if swv.size > 1:
            y = y * swv.astype(np.float64).reshape(1, -1)
        if bias is not None:
            y = y + np.asarray(bias, _F32).astype(np.float64).reshape(1, -1)
        ady = absmax(dy2, "tensor"); sdy, idy = scales_from_amax(ady)
        dyq = quantize_int(dy2, idy, "tensor", dy_round, seed, offset)
        if w_gran == "row":
            w9 = w.reshape(n * 9, c)                           # rows (n, kh, kw), columns c
            awb = absmax(w9, "col"); swb, iwb = scales_from_amax(awb)
            wqb = quantize_int(w9, iwb, "col", "nearest").reshape(n, 9 * c)
        else:
            swb, wqb = sw, wq
        acc_dx, o1 = _wrap_i32(conv3x3_dgrad_f64(dyq.reshape(b, h, wd, n), wqb.reshape(n, 3, 3, c)).reshape(m, c))
        acc_dw, o2 = _wrap_i32(conv3x3_wgrad_f64(dyq.reshape(b, h, wd, n), xq.reshape(b, h, wd, c)).reshape(n, 9 * c))
        sdyv = float(_F32(np.asarray(sdy).reshape(-1)[0]))
        swbv = np.asarray(swb, _F32).reshape(-1)
        dx = acc_dx.astype(np.float64) * sdyv
        dx = dx * (swbv.astype(np.float64).reshape(1, -1) if swbv.size > 1 else float(swbv[0]))
        dw = acc_dw.astype(np.float64) * (sdyv * sxv)
        r.update(sx=sx, sw=sw, xq=xq, wq=wq, y=y.astype(y_dtype), acc=acc, sdy=sdy, dyq=dyq, swb=swb, wqb=wqb,
                 dx=dx.astype(dx_dtype), dw=dw.astype(dw_dtype), acc_dx=acc_dx, acc_dw=acc_dw,
                 db=dy2.astype(np.float64).sum(axis=0).astype(_F32), overflow=o0 or o1 or o2)
        return r
    if tag == FP16:
        xh, wh, dyh = cast_fp16(act), cast_fp16(w), cast_fp16(dy2)
    elif tag == FP32:
        xh, wh, dyh = act.astype(_F32), w.astype(_F32), dy2.astype(_F32)
    else:
        raise ValueError(tag)
    y = conv3x3_fwd_f64(xh, wh.reshape(n, 3, 3, c)).reshape(m, n)
    if bias is not None:
        y = y + np.asarray(bias, _F32).astype(np.float64).reshape(1, -1)
    dx = conv3x3_dgrad_f64(dyh.reshape(b, h, wd, n), wh.reshape(n, 3, 3, c)).reshape(m, c)
    dw = conv3x3_wgrad_f64(dyh.reshape(b, h, wd, n), xh).reshape(n, 9 * c)
    r.update(xq=xh.reshape(m, c), wq=wh, dyq=dyh, y=y.astype(y_dtype), dx=dx.astype(dx_dtype), dw=dw.astype(dw_dtype),
             db=dy2.astype(np.float64).sum(axis=0).astype(_F32), overflow=False)
    return r
