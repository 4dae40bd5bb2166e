"""Brute-force re-derivation of the quantizer and the GEMMs in pure Python integers and Fractions.

Used only to pin the numpy oracle on tiny inputs.  Nothing here uses numpy arithmetic:
binary32 rounding is re-implemented on exact rationals, Philox on Python ints, and
the contractions are literal sums.  Written independently of ``oracle/`` on purpose.
"""
from fractions import Fraction
import math

M32 = (1 << 32) - 1


# ---------------------------------------------------------------- binary32 on rationals
def round_f32(q: Fraction) -> Fraction:
    """Nearest binary32 value (ties to even) of an exact rational, subnormals included."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()      # a ~ 2^e
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)                                               # subnormal range shares 2^-149 spacing
    ulp = Fraction(2) ** (e - 23)
    n = a / ulp
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    r = lo * ulp
    assert r < Fraction(2) ** 128, "overflow not modelled"
    return sign * r


def round_f16(q: Fraction) -> Fraction:
    """Nearest binary16 value (ties to even) of an exact rational, subnormals included; overflow not modelled."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -14)                                                # subnormal range shares 2^-24 spacing
    ulp = Fraction(2) ** (e - 10)
    n = a / ulp
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    r = lo * ulp
    assert r < Fraction(2) ** 16, "overflow not modelled"
    return sign * r


def f32_mul(a: Fraction, b: Fraction) -> Fraction:
    return round_f32(a * b)


def f32_div(a: Fraction, b: Fraction) -> Fraction:
    return round_f32(a / b)


# ------------------------------------------------------------------------------ Philox
def philox4x32_10(ctr, key):
    """ctr: four 32-bit ints (least significant word first); key: two 32-bit ints."""
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        prod_a = 0xD2511F53 * c[0]
        prod_b = 0xCD9E8D57 * c[2]
        c = [((prod_b >> 32) ^ c[1] ^ k[0]) & M32, prod_b & M32,
             ((prod_a >> 32) ^ c[3] ^ k[1]) & M32, prod_a & M32]
        k = [(k[0] + 0x9E3779B9) & M32, (k[1] + 0xBB67AE85) & M32]
    return c


def draw16(seed: int, offset: int, index: int) -> int:
    big = offset + index // 8
    ctr = [(big >> (32 * j)) & M32 for j in range(4)]
    out = philox4x32_10(ctr, [seed & M32, (seed >> 32) & M32])
    slot = index % 8
    return (out[slot // 2] >> (16 * (slot % 2))) & 0xFFFF


# ---------------------------------------------------------------------------- quantizer
def scale_pair(amax: Fraction, bits: int = 8):
    qmax = Fraction((1 << (bits - 1)) - 1)
    if amax == 0:
        return Fraction(1), Fraction(1)
    return f32_div(amax, qmax), f32_div(qmax, amax)


def quantize_scalar(x: Fraction, inv: Fraction, mode: str, u16: int = 0, bits: int = 8) -> int:
    qmax = (1 << (bits - 1)) - 1
    v = f32_mul(x, inv)
    if mode == "nearest":
        lo = math.floor(v)
        rem = v - lo
        c = lo + (1 if (rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1)) else 0)
    elif mode == "floor":
        c = math.floor(v)
    elif mode == "stochastic":
        lo = math.floor(v)
        frac = round_f32(v - lo)
        c = lo + (1 if u16 < math.floor(frac * 65536) else 0)
    else:
        raise ValueError(mode)
    return max(-qmax, min(qmax, c))


# --------------------------------------------------------------------------------- GEMM
def wrap_i32(v: int) -> int:
    v &= M32
    return v - (1 << 32) if v >= (1 << 31) else v


def gemm_nt(a, b):
    """a: list of rows [M][K], b: list of rows [N][K] -> [M][N] exact Python ints/Fractions."""
    return [[sum(ai[t] * bj[t] for t in range(len(ai))) for bj in b] for ai in a]
