"""Oracle of the general (n, p) dynamic floating-point codes (Sec. 2.1, Eq. 1-5).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``): imported by ``tests/`` alone.

A code has n bits: bit n-1 is the sign, bits n-2 .. p the exponent field e (Eq. 4; no such
field when p = n-1), bits p-1 .. 0 the significand field m.  Its integer value beta is

    sign-and-magnitude (Eq. 2):   e = 0:  (-1)^s * m                    (subnormal, step 1)
                                  e > 0:  (-1)^s * 2^(e-1) * (2^p + m)
    two's complement  (Eq. 3):    e = 0:  -s * 2^p + m
                                  e > 0:  2^(e-1) * (-s * (2^p + 2^(p+1)) + 2^p + m)

and the real value is alpha * beta (Eq. 1); here alpha = 2^-frac.  All 2^(n-1-p) exponent
codes are numbers (the paper's default: no infinities, no NaNs), so the largest value is
beta_max = 2^(2^(n-p-1) - 2) * (2^(p+1) - 1), the equality case of Eq. 5.

Readings:
* Eq. 3 prints the sign weight as the sum of 2^p and 2^(p+1) in both branches.  For e > 0 that is
  -3*2^p + 2^p = -2^(p+1), the two's complement weight of a (p+2)-bit number whose bit p is the
  hidden one; for e = 0 there is no hidden bit, and the same printed weight would leave a gap
  between -2^p and -2^(p+1): read there as -2^p (a (p+1)-bit two's complement number).
* Conversion (Sec. 3: clamp to [-gamma, gamma], divide by alpha, then rounding steps the paper does not
  spell out): gamma = alpha * beta_max; the quotient is rounded to the NEAREST representable beta, a
  tie going to the neighbour with the even significand field (IEEE 754's default, of which the
  format is declared an extension); NaN converts to 0.  The converter emits sign-and-magnitude
  codes (the symmetric set); -0 is never emitted.
"""
from __future__ import annotations

import numpy as np


def _check(n: int, p: int):
    if not (2 <= n <= 16 and 0 <= p <= n - 1 and n - 1 - p <= 5):
        raise ValueError("need 2 <= n <= 16, 0 <= p <= n-1 and at most 5 exponent bits")


def beta_max(n: int, p: int) -> int:
    """Eq. 5, equality case."""
    _check(n, p)
    if p == n - 1:
        return (1 << (n - 1)) - 1
    return (1 << ((1 << (n - p - 1)) - 2)) * ((1 << (p + 1)) - 1)


def fields(code: int, n: int, p: int):
    """(sign bit, exponent field of Eq. 4, significand field) of one code."""
    s = (code >> (n - 1)) & 1
    m = code & ((1 << p) - 1)
    e = 0 if p == n - 1 else (code >> p) & ((1 << (n - 1 - p)) - 1)
    return s, e, m


def decode(code: int, n: int, p: int) -> int:
    """Eq. 2: the integer beta of a sign-and-magnitude code."""
    _check(n, p)
    s, e, m = fields(int(code), n, p)
    mag = m if e == 0 else (1 << (e - 1)) * ((1 << p) + m)
    return -mag if s else mag


def decode_twos(code: int, n: int, p: int) -> int:
    """Eq. 3 (with the reading of its e = 0 branch stated in the module header)."""
    _check(n, p)
    s, e, m = fields(int(code), n, p)
    if e == 0:
        return -s * (1 << p) + m
    return (1 << (e - 1)) * (-s * ((1 << p) + (1 << (p + 1))) + (1 << p) + m)


def encode(beta: int, n: int, p: int) -> int:
    """The sign-and-magnitude code of a representable integer beta (inverse of Eq. 2; +0 for 0)."""
    _check(n, p)
    beta = int(beta)
    mag = abs(beta)
    s = 1 if beta < 0 else 0
    if mag < (1 << p) or p == n - 1:
        e, m = 0, mag
        if mag >= (1 << p):
            raise ValueError("not representable")
    else:
        k = mag.bit_length() - (p + 1)             # mag = 2^k * (2^p + m)
        if mag & ((1 << k) - 1) or k + 1 >= (1 << (n - 1 - p)):
            raise ValueError("not representable")
        e, m = k + 1, (mag >> k) - (1 << p)
    return (s << (n - 1)) | (e << p) | m


def round_to_beta(v, n: int, p: int) -> np.ndarray:
    """Nearest representable integer to each real v (float64 array), ties to the even significand,
    saturating at +-beta_max; NaN gives 0.  Below 2^(p+1) the representable values are the integers;
    in [2^(p+k), 2^(p+k+1)) they are the multiples of 2^k."""
    _check(n, p)
    v = np.asarray(v, np.float64)
    bm = float(beta_max(n, p))
    a = np.minimum(np.abs(np.where(np.isnan(v), 0.0, v)), bm)
    if p == n - 1:
        r = np.rint(a)                               # one binade of step 1
    else:
        _, ex = np.frexp(a)                          # a = fr * 2^ex, fr in [0.5, 1): a in [2^(ex-1), 2^ex)
        k = np.maximum(ex - 1 - p, 0)                # step 2^k
        step = np.ldexp(1.0, k)
        r = np.rint(a / step) * step                 # division by a power of two is exact; rint = ties to even
    r = np.minimum(r, bm)
    return np.where(np.signbit(v) & ~np.isnan(v), -r, r).astype(np.int64)


def quantize(x, n: int, p: int, frac: int):
    """float32 tensor -> (codes uint16, integer values int64): clamp to +-gamma = +-beta_max * 2^-frac,
    divide by alpha = 2^-frac (exact in double), round as round_to_beta, encode by Eq. 2."""
    x = np.asarray(x, np.float32)
    beta = round_to_beta(np.ldexp(x.astype(np.float64), int(frac)), n, p)
    if beta_max(n, p) >= (1 << 20):
        enc = np.frompyfunc(lambda b: encode(int(b), n, p), 1, 1)
        codes = enc(beta).astype(np.uint16) if beta.size else np.zeros(beta.shape, np.uint16)
        return codes, beta
    # formats with few integers: Eq. 2 inverted by enumerating the non-negative codes (what encode() computes, one element at a time)
    table = np.full(beta_max(n, p) + 1, -1, np.int64)
    for c in range(1 << (n - 1)):
        table[decode(c, n, p)] = c
    codes = table[np.abs(beta)] | np.where(beta < 0, 1 << (n - 1), 0)
    assert (table[np.abs(beta)] >= 0).all()
    return codes.astype(np.uint16), beta


def dequantize(codes, n: int, p: int, frac: int) -> np.ndarray:
    """codes -> float32 values alpha * beta (exact: beta has at most p+1 <= 16 significant bits)."""
    codes = np.asarray(codes)
    dec = np.frompyfunc(lambda c: decode(int(c), n, p), 1, 1)
    beta = dec(codes).astype(np.float64) if codes.size else np.zeros(codes.shape, np.float64)
    return np.ldexp(beta, -int(frac)).astype(np.float32)


def frac_from_absmax(gamma: float, n: int, p: int) -> int:
    """gamma = alpha * beta_max (Sec. 2.1) with alpha = 2^-frac: the largest frac in [-32, 32] that does not clip the
    threshold, gamma * 2^frac <= beta_max (the rule of the int8 path, applied to the format's own beta_max)."""
    _check(n, p)
    gamma = float(np.float32(gamma))
    if not (gamma >= 0.0) or np.isinf(gamma):
        raise ValueError("threshold must be finite and non-negative")
    from fractions import Fraction
    bm = beta_max(n, p)
    for f in range(32, -33, -1):
        if Fraction(gamma) * Fraction(2) ** f <= bm:
            return f
    return -32
