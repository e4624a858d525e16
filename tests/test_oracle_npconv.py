"""Pins of the oracle of the multiply-accumulate on (n, p) codes (Sec. 2.2, Eq. 6-9): brute force over Python integers
and fractions with the nearest representable value found by enumerating the whole code set, the int8 oracle (already
pinned) on the members of the family that are int8, scipy's correlation, and Eq. 8's accumulator width on the deepest
reduction of the benchmark network."""
from fractions import Fraction

import numpy as np
import pytest
import scipy.signal

import oracle
import oracle.npfmt as F
import oracle.npconv as NC


def _nearest_by_enumeration(val: Fraction, n, p):
    """The representable integer nearest to val; of two equally near ones the one whose significand field is even."""
    best = None
    for c in range(1 << n):
        b = F.decode(c, n, p)
        if b == 0 and c != 0:
            continue                      # -0
        d = abs(Fraction(b) - val)
        even = (c & 1) == 0 if p > 0 else True
        key = (d, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, b, c)
    return best[1], best[2]


CASES = [
    # fmt_x, fmt_w, fmt_y, N, H, W, C, K, R, S, stride, pad, groups, shift, relu
    ((8, 4), (8, 4), (8, 4), 1, 5, 4, 3, 4, 3, 3, 1, 1, 1, 9, False),
    ((8, 4), (8, 4), (8, 4), 2, 4, 5, 4, 2, 1, 1, 1, 0, 1, 4, True),
    ((8, 4), (8, 5), (8, 4), 1, 6, 6, 4, 4, 3, 3, 2, 1, 2, 12, False),
    ((8, 5), (8, 4), (8, 6), 1, 3, 3, 2, 3, 2, 2, 1, 0, 1, 7, True),
    ((8, 4), (8, 4), (8, 4), 1, 3, 3, 2, 2, 3, 3, 1, 1, 1, 0, False),      # no downscale: saturates almost everywhere
    ((8, 4), (8, 4), (8, 4), 1, 3, 3, 2, 2, 3, 3, 1, 1, 1, -2, False),     # upscale
    ((8, 4), (8, 4), (8, 4), 1, 4, 4, 8, 2, 3, 3, 1, 1, 1, 21, False),     # everything lands among the subnormals
    ((8, 6), (8, 7), (8, 5), 1, 4, 4, 3, 3, 3, 3, 1, 1, 1, 5, False),
]


@pytest.mark.parametrize("case", CASES)
def test_conv_np_against_integers_fractions_and_enumeration(case):
    fx, fw, fy, N, H, W, C, K, R, S, stride, pad, groups, shift, relu = case
    rng = np.random.default_rng(hash(case) & 0xffff)
    x = rng.integers(0, 256, (N, H, W, C)).astype(np.uint8)
    w = rng.integers(0, 256, (K, R, S, C // groups)).astype(np.uint8)
    b = rng.integers(-5000, 5000, K)
    y, beta, acc = NC.conv_np(x, fx, w, fw, b, shift, fy, stride, pad, groups, relu)
    bx = np.array([[[[F.decode(int(c), *fx) for c in row] for row in img] for img in n_] for n_ in x], dtype=object)
    bw = np.array([[[[F.decode(int(c), *fw) for c in row] for row in img] for img in n_] for n_ in w], dtype=object)
    P, Q = NC.out_hw(H, W, R, S, stride, pad)
    assert y.shape == (N, P, Q, K)
    for n in range(N):
        for p in range(P):
            for q in range(Q):
                for k in range(K):
                    a = NC.conv_sum_at(bx, bw, b, stride, pad, groups, n, p, q, k)
                    assert a == acc[n, p, q, k]
                    v = max(a, 0) if relu else a
                    want_b, want_c = _nearest_by_enumeration(Fraction(v, 1) / Fraction(2) ** shift, *fy)
                    assert beta[n, p, q, k] == want_b and y[n, p, q, k] == want_c, (n, p, q, k, a)


def test_ties_go_to_the_even_significand_and_saturation_is_symmetric():
    # one tap, one channel: acc = beta_x * beta_w + bias exactly; choose values that sit halfway between two codes of (8, 4)
    fy = (8, 4)
    for bxv, bwv, bias, shift, want in [(1, 1, 32, 0, 32), (1, 1, 34, 0, 36), (-1, 1, -32, 0, -32), (-1, 1, -34, 0, -36),   # step 2 above 32: 33 -> 32 (even field), 35 -> 36
                                        (3, 1, 0, 1, 2), (5, 1, 0, 1, 2), (1, 1, 0, 1, 0), (-1, 1, 0, 1, 0),                # halves among the subnormals
                                        (1984, 1984, 0, 0, 1984), (-1984, 1984, 0, 0, -1984), (1984, 1, 0, -1, 1984),      # saturation
                                        (62, 32, 0, 0, 1984), (62, 32, 32, 0, 1984),                                       # 1984 itself, and 2016: beyond the largest value
                                        (1920, 1, 32, 0, 1920), (1920, 1, 33, 0, 1984), (1920, 1, 31, 0, 1920),            # 1952: tie between 1920 (field 14) and 1984 (field 15)
                                        (1856, 1, 32, 0, 1920), (-1856, 1, -32, 0, -1920),                                 # 1888: tie between 1856 (field 13) and 1920 (field 14)
                                        (31, 31, 0, 0, 960), (31, 31, 15, 0, 960), (31, 31, 16, 0, 992)]:                  # 961 -> 960; 976 = tie of 960 (field 14) / 992 (field 15)
        x = np.array([[[[F.encode(bxv, 8, 4)]]]], np.uint8)
        w = np.array([[[[F.encode(bwv, 8, 4)]]]], np.uint8)
        y, beta, acc = NC.conv_np(x, (8, 4), w, (8, 4), np.array([bias]), shift, fy)
        assert acc[0, 0, 0, 0] == bxv * bwv + bias
        assert beta[0, 0, 0, 0] == want, (bxv, bwv, bias, shift)
        assert F.decode(int(y[0, 0, 0, 0]), *fy) == want


def test_int8_members_reduce_to_the_int8_oracle():
    """(8, 7) and (8, 6) hold the integers -127 .. 127: sum, bias, ReLU and the single rounding shift must then be what
    the int8 path's oracle (pinned on its own) computes."""
    rng = np.random.default_rng(7)
    N, H, W, C, K = 2, 6, 5, 8, 6
    xi = rng.integers(-127, 128, (N, H, W, C)).astype(np.int8)
    wi = rng.integers(-127, 128, (K, 3, 3, C // 2)).astype(np.int8)
    b = rng.integers(-3000, 3000, K).astype(np.int32)
    for fmt in [(8, 7), (8, 6)]:
        xc = np.array([F.encode(int(v), *fmt) for v in xi.ravel()], np.uint8).reshape(xi.shape)
        wc = np.array([F.encode(int(v), *fmt) for v in wi.ravel()], np.uint8).reshape(wi.shape)
        for shift, relu, stride in [(7, False, 1), (9, True, 2), (0, False, 1)]:
            y8, acc8 = oracle.conv_q(xi, wi, b, 5, shift, 5, stride=stride, pad=1, groups=2, relu=relu, want_acc=True)
            y, beta, acc = NC.conv_np(xc, fmt, wc, fmt, b, shift, fmt, stride=stride, pad=1, groups=2, relu=relu)
            assert (acc == acc8).all()
            assert (beta == y8).all()


def test_sum_is_scipys_correlation():
    rng = np.random.default_rng(11)
    bx = rng.integers(-1984, 1985, (1, 9, 8, 1))
    bw = rng.integers(-1984, 1985, (1, 3, 3, 1))
    got = NC.conv_sum(bx, bw, stride=1, pad=1)[0, :, :, 0]
    want = scipy.signal.correlate2d(bx[0, :, :, 0].astype(np.float64), bw[0, :, :, 0].astype(np.float64), mode="same")
    assert (got == want.astype(np.int64)).all()
    # stride 2, no padding: every second valid position
    got2 = NC.conv_sum(bx, bw, stride=2, pad=0)[0, :, :, 0]
    valid = scipy.signal.correlate2d(bx[0, :, :, 0].astype(np.float64), bw[0, :, :, 0].astype(np.float64), mode="valid")
    assert (got2 == valid[::2, ::2].astype(np.int64)).all()


def test_deepest_reduction_needs_eq8s_width_and_is_exact():
    """3 x 3 x 512 taps of (8, 4) codes at their extremes: Eq. 8 asks for 36 bits; the oracle must carry them."""
    bmax = F.beta_max(8, 4)
    assert bmax == 1984
    assert oracle.mac_acc_bits(3 * 3 * 512, bmax) == 36
    assert oracle.mac_max_len(32, bmax) == 545                       # Eq. 9: a 32-bit accumulator is exact for 545 terms only
    x = np.full((1, 3, 3, 512), 0x7f, np.uint8)
    w = np.stack([np.full((3, 3, 512), 0x7f, np.uint8), np.full((3, 3, 512), 0xff, np.uint8)])
    y, beta, acc = NC.conv_np(x, (8, 4), w, (8, 4), None, 25, (8, 4), stride=1, pad=1)
    assert acc[0, 1, 1, 0] == 4608 * 1984 * 1984 == -acc[0, 1, 1, 1]
    assert acc[0, 0, 0, 0] == 4 * 512 * 1984 * 1984                  # corner: four taps inside the image
    assert acc[0, 1, 1, 0] > 2 ** 34
    # 4608 * 1984^2 / 2^25 = 540.56...: between 528 (field 0 of the binade of step 32) and 544: nearest is 544
    assert beta[0, 1, 1, 0] == 544 and beta[0, 1, 1, 1] == -544


def test_eltwise_np_against_fractions_enumeration_and_the_int8_add():
    """Eq. 10 on (n, p) codes: exact rationals and the enumerated code set on random codes of mixed formats and scales;
    the members that are int8 must give what the int8 path's add (pinned on its own) gives."""
    rng = np.random.default_rng(21)
    for fa, f_a, fb, f_b, fy, f_y, relu in [((8, 4), 9, (8, 4), 9, (8, 4), 8, False), ((8, 4), 9, (8, 4), 6, (8, 4), 5, True),
                                            ((8, 4), 3, (8, 5), 12, (8, 4), 2, False), ((8, 5), 7, (8, 4), 7, (8, 6), 9, False),
                                            ((8, 4), 5, (8, 4), 5, (8, 4), 12, True), ((8, 4), 10, (8, 4), 0, (8, 4), 0, False)]:
        a = rng.integers(0, 256, 400).astype(np.uint8)
        b = rng.integers(0, 256, 400).astype(np.uint8)
        y, beta, t = NC.eltwise_np(a, fa, f_a, b, fb, f_b, fy, f_y, relu)
        for i in range(400):
            val = Fraction(F.decode(int(a[i]), *fa)) / Fraction(2) ** f_a + Fraction(F.decode(int(b[i]), *fb)) / Fraction(2) ** f_b
            if relu:
                val = max(val, Fraction(0))
            want_b, want_c = _nearest_by_enumeration(val * Fraction(2) ** f_y, *fy)
            assert beta[i] == want_b and y[i] == want_c, (i, a[i], b[i])
    ai = rng.integers(-127, 128, 2000).astype(np.int8)
    bi = rng.integers(-127, 128, 2000).astype(np.int8)
    for fmt in [(8, 7), (8, 6)]:
        ac = np.array([F.encode(int(v), *fmt) for v in ai], np.uint8)
        bc = np.array([F.encode(int(v), *fmt) for v in bi], np.uint8)
        for f_a, f_b, f_y, relu in [(4, 5, 3, True), (6, 2, 2, False), (3, 3, 3, False), (5, 4, 7, False)]:
            y8, acc8 = oracle.eltwise_q(ai, f_a, bi, f_b, f_y, relu, want_acc=True)
            _, beta, t = NC.eltwise_np(ac, fmt, f_a, bc, fmt, f_b, fmt, f_y, relu)
            assert np.array_equal(t, acc8) and np.array_equal(beta, y8)
