"""Pins of the (n, p) dynamic floating-point oracle (Sec. 2.1, Eq. 1-5) against what the paper and the
mathematics fix: Eq. 5's closed form (golden values), the code sets the paper names (Sec. 5: p = 6 is int8,
p = 2 a half-precision float cut to its top byte), IEEE binary16 as numpy implements it (the (16, 10) member of the
family without its infinities), ordinary two's complement, and the properties of round-to-nearest."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle.npfmt as F

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")
FORMATS = [(8, 7), (8, 6), (8, 5), (8, 4), (8, 3), (8, 2), (7, 3), (6, 3), (6, 4), (5, 1), (4, 0), (3, 1), (2, 1)]


def test_beta_max_is_eq5_and_the_largest_code():
    n_golden = 0
    for line in open(GOLDEN):
        parts = line.split()
        if parts and parts[0] == "beta_max":
            n, p, want = int(parts[1]), int(parts[2]), int(parts[3])
            assert F.beta_max(n, p) == want
            n_golden += 1
    assert n_golden >= 5
    for n, p in FORMATS:
        vals = [F.decode(c, n, p) for c in range(1 << n)]
        assert max(vals) == F.beta_max(n, p) == -min(vals)


@pytest.mark.parametrize("n,p", FORMATS)
def test_code_set_structure(n, p):
    """Eq. 2 + Eq. 4 over all 2^n codes: symmetric, monotone in the code, 2^p subnormal steps of 1 (Eq. 2, e = 0),
    then 2^p values per binade with the step doubling from binade to binade; no gaps between binades."""
    pos = [F.decode(c, n, p) for c in range(1 << (n - 1))]
    neg = [F.decode(c | (1 << (n - 1)), n, p) for c in range(1 << (n - 1))]
    assert neg == [-v for v in pos]
    assert pos == sorted(pos) and len(set(pos)) == len(pos) and pos[0] == 0
    assert pos[:1 << p] == list(range(1 << p))                          # subnormals: the scale alpha is the smallest positive one
    for e in range(1, 1 << (n - 1 - p)):
        binade = pos[e << p:(e + 1) << p]
        step = 1 << (e - 1)
        assert binade[0] == step << p and all(b - a == step for a, b in zip(binade, binade[1:]))
        assert binade[0] - pos[(e << p) - 1] == max(step >> 1, 1)       # the previous binade (or the subnormals) ends one of ITS steps below
    for c in range(1 << n):
        v = F.decode(c, n, p)
        if v != 0 or c == 0:
            assert F.encode(v, n, p) == c
    with pytest.raises(ValueError):
        F.encode(F.beta_max(n, p) + 1, n, p)


def test_the_formats_the_paper_names():
    # p = 6 (which Sec. 5 equates with int8) and p = n - 1: the integers -127 .. 127, sign and magnitude
    for p in (6, 7):
        assert sorted(F.decode(c, 8, p) for c in range(256)) == sorted(list(range(-127, 128)) + [0])
    # Eq. 3 with p = n - 1 is ordinary two's complement
    assert [F.decode_twos(c, 8, 7) for c in range(256)] == np.arange(256, dtype=np.uint8).view(np.int8).tolist()
    # p = 2 (Sec. 5: a truncated half-precision float): the top byte of an IEEE binary16, scaled by 2^16; and (16, 10) IS binary16
    # scaled by 2^24 - on every code that binary16 does not spend on infinities and NaNs
    for c in range(256):
        if (c >> 2) & 31 != 31:
            assert Fraction(F.decode(c, 8, 2), 2 ** 16) == Fraction(float(np.array([c << 8], np.uint16).view(np.float16)[0]))
    for c in list(range(0, 1 << 16, 7)) + [0x7bff, 0xfbff, 0x0001, 0x8001, 0x03ff, 0x0400]:
        if (c >> 10) & 31 != 31:
            assert Fraction(F.decode(c, 16, 10), 2 ** 24) == Fraction(float(np.array([c], np.uint16).view(np.float16)[0]))
    # the all-ones exponent holds numbers, not infinities: one more binade above binary16's largest finite value
    assert F.decode(0x7c00, 16, 10) == 2 ** 30 * 1024 and F.decode(0x7fff, 16, 10) == F.beta_max(16, 10)
    # Eq. 3, e > 0: negative codes mirror the positive binade one step further out (as -128 does for int8)
    n, p = 8, 4
    for e in range(1, 8):
        negs = sorted(F.decode_twos((1 << 7) | (e << p) | m, n, p) for m in range(16))
        assert negs == [-(1 << (e - 1)) * k for k in range(32, 16, -1)]
    assert [F.decode_twos((1 << 7) | m, n, p) for m in range(16)] == list(range(-16, 0))       # e = 0: (p+1)-bit two's complement


def test_conversion_is_numpys_binary16_rounding_for_16_10():
    """quantize(x, 16, 10, 24) must produce the bits numpy's float32 -> float16 conversion produces (round to nearest,
    ties to even, gradual underflow) wherever binary16 has not overflowed: an independent implementation of the same
    rounding."""
    rng = np.random.default_rng(9)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-8, 5, 20000).astype(np.float32),
                        np.array([0.0, 1.0, 65504.0, 65519.9, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, 1.0 + 2.0 ** -11,
                                  1.0 + 3 * 2.0 ** -11, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25], np.float32)])
    x = np.concatenate([x, -x])
    codes, beta = F.quantize(x, 16, 10, 24)
    h = x.astype(np.float16)
    ok = np.isfinite(h)
    assert ok.sum() > 30000
    want = h.view(np.uint16)
    nz = ok & (beta != 0)                                  # the oracle never emits -0
    assert np.array_equal(codes[nz], want[nz])
    assert np.all((want[ok & (beta == 0)] & 0x7fff) == 0)
    assert np.array_equal(F.dequantize(codes[ok], 16, 10, 24), h[ok].astype(np.float32))


@pytest.mark.parametrize("n,p", [(8, 4), (8, 3), (8, 2), (6, 3), (8, 7), (5, 1)])
def test_conversion_properties(n, p):
    """Nearest representable value (exact rational check of the half-step bound and of ties), saturation at
    gamma = alpha * beta_max, odd symmetry, monotonicity, idempotence, NaN -> 0, Inf -> +-gamma."""
    rng = np.random.default_rng(100 * n + p)
    frac = 3
    bm = F.beta_max(n, p)
    gamma = bm / 2.0 ** frac
    x = (rng.standard_normal(4000) * gamma / 3).astype(np.float32)
    x[:200] = (rng.standard_normal(200) * 4.0 / 2 ** frac).astype(np.float32)        # subnormal range
    codes, beta = F.quantize(x, n, p, frac)
    reps = sorted(F.decode(c, n, p) for c in range(1 << (n - 1)))
    for xi, bi in zip(x[:600].tolist(), beta[:600].tolist()):
        v = Fraction(xi) * 2 ** frac
        if abs(v) >= bm:
            assert bi == (bm if v > 0 else -bm)
            continue
        best = min(abs(Fraction(r) - abs(v)) for r in reps)
        assert abs(Fraction(abs(bi)) - abs(v)) == best and (bi == 0 or (bi > 0) == (v > 0))
    # ties go to the even significand: halfway between neighbours r0 < r1 the result is the one whose code is even
    for i in range(0, len(reps) - 1, max(1, len(reps) // 40)):
        r0, r1 = reps[i], reps[i + 1]
        mid = np.array([(r0 + r1) / 2.0 / 2 ** frac], np.float32)
        got = int(F.quantize(mid, n, p, frac)[1][0])
        want = r0 if F.encode(r0, n, p) % 2 == 0 else r1
        assert got == want, (r0, r1)
    c2, b2 = F.quantize(-x, n, p, frac)
    assert np.array_equal(b2, -beta)
    xs = np.sort(x)
    assert np.all(np.diff(F.quantize(xs, n, p, frac)[1]) >= 0)
    assert np.array_equal(F.quantize(F.dequantize(codes, n, p, frac), n, p, frac)[0], codes)
    sp = np.array([np.nan, np.inf, -np.inf, 1e30, -1e30, 0.0, -0.0], np.float32)
    assert F.quantize(sp, n, p, frac)[1].tolist() == [0, bm, -bm, bm, -bm, 0, 0]
    assert F.dequantize(F.quantize(sp, n, p, frac)[0], n, p, frac).tolist() == [0.0, gamma, -gamma, gamma, -gamma, 0.0, 0.0]
    # every code survives the round trip through float (the codes of -0 aside)
    allc = np.array([c for c in range(1 << n) if c != 1 << (n - 1)], np.uint16)
    assert np.array_equal(F.quantize(F.dequantize(allc, n, p, frac), n, p, frac)[0], allc)


def test_int8_member_agrees_with_the_int8_oracle():
    """(8, 7) through the general converter gives the codes of the int8 path (sign and magnitude vs two's complement aside)."""
    import oracle as orc
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(5000) * 3).astype(np.float32)
    for f in (0, 4, 7):
        assert np.array_equal(F.quantize(x, 8, 7, f)[1], orc.quantize(x, f).astype(np.int64))
        assert np.array_equal(F.quantize(x, 8, 6, f)[1], orc.quantize(x, f).astype(np.int64))


def test_frac_from_absmax_hand_values_and_the_int8_rule():
    """The threshold-to-scale rule on the general family: hand-worked values, the int8 path's rule (pinned on its own) for
    the member that is int8, and the two properties that define it (the threshold is not clipped; one more bit would clip)."""
    import oracle
    assert F.frac_from_absmax(1984.0, 8, 4) == 0 and F.frac_from_absmax(1985.0, 8, 4) == -1
    assert F.frac_from_absmax(1.0, 8, 4) == 10            # 1024 <= 1984 < 2048
    assert F.frac_from_absmax(3.9, 8, 4) == 8             # 3.9 * 512 = 1996.8 is too much
    assert F.frac_from_absmax(0.0, 8, 4) == 32 and F.frac_from_absmax(1e30, 8, 4) == -32
    assert F.frac_from_absmax(0.25, 8, 3) == 19           # beta_max(8, 3) = 245760 = 0.46875 * 2^19
    rng = np.random.default_rng(5)
    for g in np.exp(rng.uniform(-15, 15, 300)).astype(np.float32):
        assert F.frac_from_absmax(g, 8, 7) == oracle.frac_from_absmax_f32(float(g))
        for n, p in [(8, 4), (8, 3), (6, 2)]:
            f = F.frac_from_absmax(g, n, p)
            bm = F.beta_max(n, p)
            if -32 < f:
                assert Fraction(float(g)) * Fraction(2) ** f <= bm
            if f < 32:
                assert Fraction(float(g)) * Fraction(2) ** (f + 1) > bm
    with pytest.raises(ValueError):
        F.frac_from_absmax(float("nan"), 8, 4)
