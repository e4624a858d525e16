"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here re-types the oracle's formulas: expected values are hand-worked
closed-form numbers (tests/golden/closed_forms.txt), exact rational arithmetic
with ``fractions.Fraction`` / Python big integers, brute-force enumeration, or
library routines (numpy int64 matmul, scipy correlate2d) for special cases.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.signal import correlate2d

import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


def _golden():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            parts = line.split()
            rows.append((parts[0], [int(v) for v in parts[1:]]))
    return rows


# --------------------------------------------------------------------------- #
# Sec. 2.1 / 2.2 closed forms                                                   #
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("kind,vals", _golden())
def test_closed_forms_golden(kind, vals):
    *args, want = vals
    fn = {"beta_max": orc.beta_max, "mac_bits": orc.mac_acc_bits, "mac_len": orc.mac_max_len,
          "add_bits": orc.add_acc_bits, "add_len": orc.add_max_len}[kind]
    assert fn(*args) == want


def _decode_sign_magnitude(bits, n, p):
    """Eq. 2 with Eq. 4, by enumeration of the bit pattern."""
    b = [(bits >> i) & 1 for i in range(n)]
    e_hat = 0 if p == n - 1 else sum(b[i] << (i - p) for i in range(p, n - 1))
    m = sum(b[i] << i for i in range(p))
    sign = -1 if b[n - 1] else 1
    if e_hat == 0:
        return sign * m
    return sign * (2 ** (e_hat - 1)) * (2 ** p + m)


@pytest.mark.parametrize("n,p", [(8, 7), (8, 6), (8, 5), (8, 4), (8, 3), (7, 3), (6, 3), (6, 2), (5, 1), (4, 0)])
def test_beta_max_is_largest_decoded_code(n, p):
    codes = [_decode_sign_magnitude(v, n, p) for v in range(2 ** n)]
    assert max(codes) == orc.beta_max(n, p)
    assert min(codes) == -orc.beta_max(n, p)          # sign-magnitude range is symmetric


def test_int8_member_of_family_has_every_integer_code():
    # p = n-1 = 7 and p = 6 both give exactly the integers -127..127
    for p in (7, 6):
        assert sorted(set(_decode_sign_magnitude(v, 8, p) for v in range(256))) == list(range(-127, 128))


def _smallest_q(lo, hi):
    q = 1
    while not (-(2 ** (q - 1)) <= lo and hi <= 2 ** (q - 1) - 1):
        q += 1
    return q


def test_mac_width_is_smallest_accumulator_that_holds_eq7_range():
    for N, bx, ex, by, ey in itertools.product([1, 2, 3, 7, 64, 576, 4608], [1, 7, 127], [0, 1, 3], [1, 15, 127], [0, 1]):
        ax, ay = -bx - ex, -by - ey
        lo = N * min(ay * bx, ax * by)
        hi = N * ax * ay
        assert orc.mac_acc_bits(N, bx, ex, by, ey) == _smallest_q(lo, hi), (N, bx, ex, by, ey)


def test_mac_len_is_largest_n_for_width():
    for q, bx, ex, by, ey in itertools.product([9, 16, 24, 32], [7, 127], [0, 1], [15, 127], [0, 1]):
        N = orc.mac_max_len(q, bx, ex, by, ey)
        hi = lambda n: n * (bx + ex) * (by + ey)
        assert hi(N) <= 2 ** (q - 1) - 1 < hi(N + 1)


def test_add_width_and_length():
    for N, bx, ex in itertools.product([1, 2, 3, 49, 1000], [1, 7, 127], [0, 1, 2]):
        assert orc.add_acc_bits(N, bx, ex) == _smallest_q(N * (-bx - ex), N * bx), (N, bx, ex)
    for q, bx, ex in itertools.product([8, 9, 14, 16, 32], [7, 127], [0, 1, 2]):
        N = orc.add_max_len(q, bx, ex)
        fits = lambda n: -(2 ** (q - 1)) <= n * (-bx - ex) and n * bx <= 2 ** (q - 1) - 1
        assert fits(N) and not fits(N + 1)


def test_int32_accumulator_suffices_for_every_layer_of_the_configs():
    # deepest reduction in the five configs is 3x3x512 = 4608 products of codes that may reach -128
    assert orc.mac_acc_bits(4608, 127, 1, 127, 1) <= 32
    assert orc.mac_max_len(32, 127, 1, 127, 1) >= 4608


# --------------------------------------------------------------------------- #
# rounding                                                                      #
# --------------------------------------------------------------------------- #

def _round_even(fr: Fraction) -> int:
    return round(fr)  # Python rounds a Fraction to the nearest integer, ties to even


def _sat(v):
    return max(-127, min(127, v))


def test_rne_shift_matches_exact_rational_rounding():
    rng = np.random.default_rng(1)
    vals = list(range(-70, 71)) + [int(v) for v in rng.integers(-2 ** 31, 2 ** 31, 4000)]
    for v in vals:
        for s in (0, 1, 2, 3, 5, 7, 8, 13, 20, 31, 32, 40):
            assert orc.rne_shift(v, s) == _round_even(Fraction(v, 2 ** s)), (v, s)
        for s in (-1, -3, -8):
            assert orc.rne_shift(v, s) == v * 2 ** (-s)


def test_rne_ties_by_hand():
    # value/2: 1/2 -> 0, 3/2 -> 2, 5/2 -> 2, -1/2 -> 0, -3/2 -> -2, -5/2 -> -2
    assert [orc.rne_shift(v, 1) for v in (1, 3, 5, -1, -3, -5)] == [0, 2, 2, 0, -2, -2]
    # value/4: 2/4 -> 0, 6/4 -> 2, 10/4 -> 2, 5/4 -> 1, 7/4 -> 2
    assert [orc.rne_shift(v, 2) for v in (2, 6, 10, 5, 7)] == [0, 2, 2, 1, 2]


def test_requant8_any_shift():
    rng = np.random.default_rng(2)
    for v in [0, 1, -1, 127, -128, 2 ** 31 - 1, -2 ** 31] + [int(t) for t in rng.integers(-2 ** 31, 2 ** 31, 500)]:
        for s in range(-100, 101):
            want = _sat(_round_even(Fraction(v) / Fraction(2) ** s))
            assert orc.requant8(v, s) == want, (v, s)


# --------------------------------------------------------------------------- #
# float <-> code                                                                #
# --------------------------------------------------------------------------- #

def test_quantize_hand_values():
    x = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 0.49999997, 126.5, 127.5, 300.0, -300.0,
                  np.inf, -np.inf, np.nan, -128.0, 127.49], np.float32)
    want = [0, 2, 2, 0, -2, -2, 0, 126, 127, 127, -127, 127, -127, 0, -127, 127]
    assert orc.quantize(x, 0).tolist() == want
    assert orc.quantize(np.array([0.03125, 0.09375, 1.0, -1.0, 7.9375, 8.0], np.float32), 4).tolist() == \
        [0, 2, 16, -16, 127, 127]
    assert orc.quantize(np.array([96.0, 160.0, 1000.0, 1e9], np.float32), -6).tolist() == [2, 2, 16, 127]


def test_quantize_matches_exact_rational_rounding_and_properties():
    rng = np.random.default_rng(3)
    for f in (-6, -1, 0, 3, 4, 7, 12):
        x = (rng.standard_normal(3000) * 2.0 ** (-f + 5)).astype(np.float32)
        ties = ((rng.integers(-300, 300, 400) + 0.5) * 2.0 ** -f).astype(np.float32)
        x = np.concatenate([x, ties])
        q = orc.quantize(x, f)
        want = [_sat(_round_even(Fraction(float(v)) * Fraction(2) ** f)) for v in x]
        assert q.tolist() == want
        # odd symmetry: fails for an asymmetric clamp or for round-half-up
        assert np.array_equal(orc.quantize(-x, f), -q)
        # monotone
        order = np.argsort(x, kind="stable")
        assert np.all(np.diff(q[order].astype(np.int32)) >= 0)
        # round trip: |x - dq(q(x))| <= half a step inside the range
        inside = np.abs(x) <= 127 * 2.0 ** -f
        err = np.abs(x.astype(np.float64) - orc.dequantize(q, f).astype(np.float64))
        assert np.all(err[inside] <= 2.0 ** -(f + 1))
        # idempotent on codes; -128 is never produced
        codes = np.arange(-127, 128).astype(np.int8)
        assert np.array_equal(orc.quantize(orc.dequantize(codes, f), f), codes)
        assert q.min() >= -127


def test_dequantize_is_exact_scaling():
    codes = np.arange(-128, 128).astype(np.int8)
    for f in (-32, -3, 0, 4, 7, 32):
        got = orc.dequantize(codes, f)
        want = np.array([float(Fraction(int(c)) / Fraction(2) ** f) for c in codes], np.float32)
        assert np.array_equal(got, want)


def test_quantize_i32_saturates_and_rounds():
    x = np.array([0.5, 1.5, -2.5, 3e9, -3e9, 2147483520.0, np.nan, 0.1], np.float32)
    assert orc.quantize_i32(x, 0).tolist() == [0, 2, -2, 2 ** 31 - 1, -(2 ** 31 - 1), 2147483520, 0, 0]
    assert orc.quantize_i32(np.array([0.1], np.float32), 11).tolist() == \
        [_round_even(Fraction(float(np.float32(0.1))) * 2 ** 11)]


# --------------------------------------------------------------------------- #
# convolution                                                                   #
# --------------------------------------------------------------------------- #

def _brute_conv(x, w, b, stride, pad, groups):
    """Independent big-int statement of the convolution sum over *padded* input."""
    N, H, W, C = x.shape
    K, R, S, Cg = w.shape
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C), dtype=object)
    xp[:, pad:pad + H, pad:pad + W, :] = x.astype(object)
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    Kg = K // groups
    out = np.zeros((N, P, Q, K), dtype=object)
    for n, p, q, k in itertools.product(range(N), range(P), range(Q), range(K)):
        g = k // Kg
        patch = xp[n, p * stride:p * stride + R, q * stride:q * stride + S, g * Cg:(g + 1) * Cg]
        out[n, p, q, k] = int((patch * w[k].astype(object)).sum()) + (0 if b is None else int(b[k]))
    return out


CONV_CASES = [
    # N  H  W  C  K  R  S  st pad groups
    (1, 5, 5, 3, 4, 3, 3, 1, 1, 1),
    (2, 6, 5, 4, 6, 3, 3, 2, 1, 2),
    (1, 7, 7, 2, 2, 5, 5, 1, 2, 1),
    (1, 8, 6, 6, 6, 3, 3, 2, 0, 6),
    (2, 4, 4, 8, 3, 1, 1, 1, 0, 1),
    (1, 9, 9, 3, 5, 7, 7, 2, 3, 1),
    (1, 3, 4, 4, 8, 2, 3, 1, 1, 4),
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_matches_bigint_brute_force(case):
    N, H, W, C, K, R, S, st, pad, g = case
    rng = np.random.default_rng(sum(case))
    x = rng.integers(-128, 128, (N, H, W, C)).astype(np.int8)
    w = rng.integers(-128, 128, (K, R, S, C // g)).astype(np.int8)
    b = rng.integers(-2 ** 20, 2 ** 20, (K,)).astype(np.int32)
    want = _brute_conv(x, w, b, st, pad, g)
    for f_in, f_w, f_out, relu in [(4, 7, 4, 0), (4, 7, 4, 1), (3, 5, 8, 0), (2, 2, 9, 1), (5, 6, -2, 0)]:
        y, acc = orc.conv_q(x, w, b, f_in, f_w, f_out, st, pad, g, relu, want_acc=True)
        assert np.array_equal(acc.astype(object), want)
        ref = np.vectorize(lambda a: _sat(_round_even(Fraction(max(a, 0) if relu else a) /
                                                      Fraction(2) ** (f_in + f_w - f_out))))(want)
        assert np.array_equal(y.astype(np.int64), ref.astype(np.int64))
    # no bias
    _, acc = orc.conv_q(x, w, None, 0, 0, 0, st, pad, g, 0, want_acc=True)
    assert np.array_equal(acc.astype(object), _brute_conv(x, w, None, st, pad, g))
    # single-element entry point agrees
    P, Q = acc.shape[1:3]
    for n, p, q, k in [(0, 0, 0, 0), (N - 1, P - 1, Q - 1, K - 1), (0, P // 2, Q // 2, K // 2)]:
        assert orc.conv_acc_at(x, w, b, st, pad, g, n, p, q, k) == want[n, p, q, k]


def test_conv_1x1_is_an_integer_matrix_product():
    rng = np.random.default_rng(5)
    x = rng.integers(-128, 128, (2, 5, 7, 40)).astype(np.int8)
    w = rng.integers(-128, 128, (24, 1, 1, 40)).astype(np.int8)
    b = rng.integers(-1000, 1000, 24).astype(np.int32)
    _, acc = orc.conv_q(x, w, b, 0, 0, 0, want_acc=True)
    want = x.reshape(-1, 40).astype(np.int64) @ w.reshape(24, 40).astype(np.int64).T + b
    assert np.array_equal(acc.reshape(-1, 24), want)
    # stride 2 on a 1x1 kernel just subsamples the pixels
    _, acc2 = orc.conv_q(x, w, b, 0, 0, 0, stride=2, want_acc=True)
    assert np.array_equal(acc2, acc[:, ::2, ::2, :])


def test_depthwise_is_per_channel_2d_correlation():
    rng = np.random.default_rng(6)
    C = 5
    x = rng.integers(-128, 128, (1, 9, 8, C)).astype(np.int8)
    w = rng.integers(-128, 128, (C, 3, 3, 1)).astype(np.int8)
    _, acc = orc.conv_q(x, w, None, 0, 0, 0, stride=1, pad=1, groups=C, want_acc=True)
    for c in range(C):
        want = correlate2d(x[0, :, :, c].astype(np.int64), w[c, :, :, 0].astype(np.int64), mode="same")
        assert np.array_equal(acc[0, :, :, c], want)


def test_grouped_equals_dense_with_block_diagonal_weights():
    rng = np.random.default_rng(7)
    g, Cg, Kg = 3, 4, 2
    x = rng.integers(-128, 128, (2, 6, 6, g * Cg)).astype(np.int8)
    w = rng.integers(-128, 128, (g * Kg, 3, 3, Cg)).astype(np.int8)
    dense = np.zeros((g * Kg, 3, 3, g * Cg), np.int8)
    for k in range(g * Kg):
        gi = k // Kg
        dense[k, :, :, gi * Cg:(gi + 1) * Cg] = w[k]
    ya, acca = orc.conv_q(x, w, None, 3, 6, 2, 2, 1, g, 1, want_acc=True)
    yb, accb = orc.conv_q(x, dense, None, 3, 6, 2, 2, 1, 1, 1, want_acc=True)
    assert np.array_equal(acca, accb) and np.array_equal(ya, yb)


def test_extreme_codes_reach_the_eq8_bound_exactly():
    x = np.full((1, 3, 3, 512), -128, np.int8)
    w = np.full((1, 3, 3, 512), -128, np.int8)
    _, acc = orc.conv_q(x, w, None, 0, 0, 0, want_acc=True)
    assert acc.shape == (1, 1, 1, 1) and int(acc[0, 0, 0, 0]) == 4608 * 16384 == 75497472
    assert 75497472 < 2 ** (orc.mac_acc_bits(4608, 127, 1, 127, 1) - 1)


def test_conv_reports_int32_overflow():
    x = np.full((1, 1, 1, 8), -128, np.int8)
    w = np.full((1, 1, 1, 8), -128, np.int8)
    b = np.array([2 ** 31 - 1], np.int32)
    with pytest.raises(OverflowError):
        orc.conv_q(x, w, b, 0, 0, 0)


def test_relu_commutes_with_requantize():
    rng = np.random.default_rng(8)
    x = rng.integers(-128, 128, (1, 6, 6, 8)).astype(np.int8)
    w = rng.integers(-128, 128, (8, 3, 3, 8)).astype(np.int8)
    for s_out in (0, 3, 9, 12):
        y_relu, _ = orc.conv_q(x, w, None, 4, 7, s_out, 1, 1, 1, relu=True)
        y_lin, _ = orc.conv_q(x, w, None, 4, 7, s_out, 1, 1, 1, relu=False)
        assert np.array_equal(y_relu, np.maximum(y_lin, 0))


def test_identity_convolution_is_the_explicit_downscale():
    rng = np.random.default_rng(9)
    C = 6
    x = rng.integers(-127, 128, (2, 4, 5, C)).astype(np.int8)
    for f_w in (0, 3, 6):
        w = (np.eye(C, dtype=np.int64) * 2 ** f_w).astype(np.int8).reshape(C, 1, 1, C)
        y, _ = orc.conv_q(x, w, None, 4, f_w, 4)
        assert np.array_equal(y, x)                       # factor 1: the layer could be spliced out
        for f_out in (3, 1, -2):
            y, _ = orc.conv_q(x, w, None, 4, f_w, f_out)
            assert np.array_equal(y, orc.concat_q([x], [4], f_out))
            z, _ = orc.eltwise_q(x, 4, np.zeros_like(x), 4, f_out)
            assert np.array_equal(y, z)
            want = np.vectorize(lambda c: _sat(_round_even(Fraction(int(c), 2 ** (4 - f_out)))))(x)
            assert np.array_equal(y.astype(np.int64), want)


# --------------------------------------------------------------------------- #
# joins and pooling                                                             #
# --------------------------------------------------------------------------- #

def test_eltwise_is_one_rounding_of_the_exact_sum():
    codes = np.arange(-128, 128).astype(np.int8)
    a, b = np.meshgrid(codes, codes, indexing="ij")
    a, b = a.ravel(), b.ravel()
    for fa, fb, fy, relu in [(4, 4, 4, 0), (4, 4, 3, 1), (5, 2, 3, 0), (2, 6, 1, 1), (3, 4, 5, 0), (0, 7, -1, 0), (-3, -1, -4, 1)]:
        y, acc = orc.eltwise_q(a, fa, b, fb, fy, relu, want_acc=True)
        exact = [Fraction(int(u), 1) / Fraction(2) ** fa + Fraction(int(v), 1) / Fraction(2) ** fb for u, v in zip(a, b)]
        F = max(fa, fb)
        assert acc.tolist() == [int(e * Fraction(2) ** F) for e in exact]
        want = [_sat(_round_even((max(e, 0) if relu else e) * Fraction(2) ** fy)) for e in exact]
        assert y.tolist() == want
        y2, _ = orc.eltwise_q(b, fb, a, fa, fy, relu)
        assert np.array_equal(y, y2)                      # commutative
    y, _ = orc.eltwise_q(a, 4, b, 4, 4)
    assert np.array_equal(y, np.clip(a.astype(np.int32) + b, -127, 127))
    with pytest.raises(ValueError):
        orc.eltwise_q(a, 30, b, 0, 0)


def test_eltwise_is_a_special_mac():
    # add = 1x1 convolution over channel-stacked inputs with power-of-two "weights" (Sec. 2.2, first paragraph)
    rng = np.random.default_rng(10)
    C = 5
    a = rng.integers(-128, 128, (1, 4, 4, C)).astype(np.int8)
    b = rng.integers(-128, 128, (1, 4, 4, C)).astype(np.int8)
    fa, fb, fy = 3, 5, 2
    F = max(fa, fb)
    w = np.concatenate([np.eye(C, dtype=np.int64) * 2 ** (F - fa), np.eye(C, dtype=np.int64) * 2 ** (F - fb)], axis=1)
    w = w.astype(np.int8).reshape(C, 1, 1, 2 * C)
    # inputs at a common nominal f_in = 0 with weights at f_w = F  ->  accumulator is the sum at F
    y_conv, _ = orc.conv_q(np.concatenate([a, b], axis=3), w, None, 0, F, fy, relu=True)
    y_add, _ = orc.eltwise_q(a, fa, b, fb, fy, relu=True)
    assert np.array_equal(y_conv, y_add)


def test_concat_rescales_each_branch_on_its_own():
    rng = np.random.default_rng(11)
    xs = [rng.integers(-128, 128, (2, 3, 3, c)).astype(np.int8) for c in (3, 1, 4)]
    fs = [5, 2, 3]
    y = orc.concat_q(xs, fs, 2)
    assert y.shape == (2, 3, 3, 8)
    off = 0
    for x, f in zip(xs, fs):
        want = np.vectorize(lambda c: _sat(_round_even(Fraction(int(c), 2 ** (f - 2)))))(x)
        assert np.array_equal(y[..., off:off + x.shape[-1]].astype(np.int64), want)
        off += x.shape[-1]
    # equal formats: a byte copy, except that -128 is clamped into the symmetric range
    y = orc.concat_q(xs, [3, 3, 3], 3)
    assert np.array_equal(y, np.maximum(np.concatenate(xs, axis=3), -127))
    # finer output format: exact multiplication then clamp
    y = orc.concat_q([xs[0]], [2], 4)
    assert np.array_equal(y, np.clip(xs[0].astype(np.int32) * 4, -127, 127))


def _pool_ref(x, mode, k, st, pad, d):
    N, H, W, C = x.shape
    P, Q = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    out = np.zeros((N, P, Q, C), np.int64)
    for n, p, q, c in itertools.product(range(N), range(P), range(Q), range(C)):
        vals = [int(x[n, ih, iw, c]) for ih in range(p * st - pad, p * st - pad + k)
                for iw in range(q * st - pad, q * st - pad + k) if 0 <= ih < H and 0 <= iw < W]
        if mode == "max":
            out[n, p, q, c] = _sat(_round_even(Fraction(max(vals)) * Fraction(2) ** d))
        else:
            out[n, p, q, c] = _sat(_round_even(Fraction(sum(vals), k * k) * Fraction(2) ** d))
    return out


@pytest.mark.parametrize("mode", ["max", "avg"])
def test_pool_matches_exact_rational_reference(mode):
    rng = np.random.default_rng(12)
    x = rng.integers(-128, 128, (2, 7, 6, 3)).astype(np.int8)
    for k, st, pad in [(3, 2, 1), (3, 1, 1), (2, 2, 0), (7, 1, 3), (1, 1, 0), (6, 1, 0)]:
        if k > 6 and pad == 0:
            continue
        for f_in, f_out in [(4, 4), (4, 2), (3, 5), (0, -3)]:
            got = orc.pool_q(x, mode, k, st, pad, f_in, f_out)
            assert np.array_equal(got.astype(np.int64), _pool_ref(x, mode, k, st, pad, f_out - f_in)), (k, st, pad, f_in, f_out)


def test_pool_special_cases():
    rng = np.random.default_rng(13)
    x = rng.integers(-127, 128, (1, 6, 6, 4)).astype(np.int8)
    for mode in ("max", "avg"):
        assert np.array_equal(orc.pool_q(x, mode, 1, 1, 0, 3, 3), x)                 # k = 1 is the identity
        const = np.full((1, 6, 6, 4), -37, np.int8)
        assert np.all(orc.pool_q(const, mode, 3, 3, 0, 3, 3) == -37)                  # constant stays constant
    # max commutes with the (monotone) rescale
    a = orc.pool_q(orc.concat_q([x], [5], 2), "max", 3, 2, 1, 2, 2)
    b = orc.pool_q(x, "max", 3, 2, 1, 5, 2)
    assert np.array_equal(a, b)
    # global average equals numpy's mean rounded half-even (exact rational compare)
    g = orc.pool_q(x, "avg", 6, 1, 0, 3, 3)
    want = [_sat(_round_even(Fraction(int(x[0, :, :, c].astype(np.int64).sum()), 36))) for c in range(4)]
    assert g.reshape(-1).tolist() == want
    # a 7x7 window of symmetric codes fits Eq. 12's 14-bit accumulator
    assert 49 * 127 <= 2 ** (orc.add_acc_bits(49, 127) - 1) - 1


# --------------------------------------------------------------------------- #
# calibration building blocks                                                   #
# --------------------------------------------------------------------------- #

def test_format_from_float_threshold():
    f = orc.frac_from_absmax_f32
    assert f(1.0) == 6            # 127/64 = 1.98 >= 1 but 127/128 < 1
    assert f(1.99) == 5
    assert f(0.0) == 32
    for k in range(-10, 11):
        assert f(127.0 * 2.0 ** -k) == k
        assert f(float(np.nextafter(np.float32(127.0 * 2.0 ** -k), np.float32(np.inf)))) == k - 1
    assert f(1e30) == -32
    with pytest.raises(ValueError):
        f(float("nan"))
    # gamma = alpha * beta_max: the chosen scale is the smallest power of two that still holds gamma
    rng = np.random.default_rng(14)
    for g in np.abs(rng.standard_normal(200)).astype(np.float32) * 50:
        k = f(float(g))
        assert Fraction(float(g)) * Fraction(2) ** k <= 127 < Fraction(float(g)) * Fraction(2) ** (k + 1)


def test_format_from_integer_threshold():
    f = orc.frac_from_absmax_i32
    assert f(0, 11) == 11
    assert f(127, 11) == 11
    assert f(128, 11) == 10
    assert f(254, 11) == 10
    assert f(255, 11) == 9
    assert f(127 * 2 ** 7, 11) == 4
    assert f(127 * 2 ** 7 + 1, 11) == 3
    assert f(1, 40) == 32
    rng = np.random.default_rng(15)
    for m in [int(v) for v in rng.integers(1, 2 ** 31, 300)]:
        for af in (-5, 0, 9, 13):
            k = f(m, af)
            assert k <= af
            assert Fraction(m) / Fraction(2) ** (af - k) <= 127                     # nothing is clipped
            if k < af:
                assert Fraction(m) / Fraction(2) ** (af - k - 1) > 127              # and no bit is wasted


def test_absmax():
    assert orc.absmax_f32(np.array([0.5, -3.25, np.nan, 2.0], np.float32)) == 3.25
    a = np.array([5, -9, 3, -(2 ** 31)], np.int32)
    assert orc.absmax_i32(a) == 2 ** 31
    assert orc.absmax_i32(a, relu=True) == 5
    assert orc.absmax_i32(np.zeros(4, np.int32)) == 0


def test_requant_i32_is_the_last_step_of_conv():
    rng = np.random.default_rng(16)
    x = rng.integers(-128, 128, (1, 6, 6, 8)).astype(np.int8)
    w = rng.integers(-128, 128, (8, 3, 3, 8)).astype(np.int8)
    b = rng.integers(-5000, 5000, 8).astype(np.int32)
    for f_out, relu in [(4, 0), (2, 1), (12, 0), (-1, 1)]:
        y, acc = orc.conv_q(x, w, b, 4, 7, f_out, 1, 1, 1, relu, want_acc=True)
        assert np.array_equal(orc.requant_i32(acc, 11 - f_out, relu), y)
        want = [_sat(_round_even(Fraction(max(int(v), 0) if relu else int(v)) / Fraction(2) ** (11 - f_out)))
                for v in acc.ravel()]
        assert y.ravel().tolist() == want


# --------------------------------------------------------------------------- #
# One weight format per output channel (Sec. 3: weight thresholds are taken per output channel)
# --------------------------------------------------------------------------- #

@pytest.mark.parametrize("case", CONV_CASES)
def test_per_channel_conv_matches_exact_rational_rescale(case):
    """Channel k's accumulator stands for acc * 2^-(f_in + f_w[k]); the output is that value rounded
    once (ties to even) onto the grid of f_out and clamped - evaluated here with big ints and Fractions."""
    N, H, W, C, K, R, S, st, pad, g = case
    rng = np.random.default_rng(1000 + sum(case))
    x = rng.integers(-128, 128, (N, H, W, C)).astype(np.int8)
    w = rng.integers(-128, 128, (K, R, S, C // g)).astype(np.int8)
    b = rng.integers(-2 ** 20, 2 ** 20, (K,)).astype(np.int32)
    want = _brute_conv(x, w, b, st, pad, g)
    for f_in, f_out, relu in [(4, 4, 0), (3, 6, 1), (5, -2, 0)]:
        f_w = rng.integers(2, 12, K).astype(np.int32)
        y, acc = orc.conv_q(x, w, b, f_in, f_w, f_out, st, pad, g, relu, want_acc=True)
        assert np.array_equal(acc.astype(object), want)
        for k in range(K):
            ref = np.vectorize(lambda a: _sat(_round_even(Fraction(max(a, 0) if relu else a) * Fraction(2) ** f_out /
                                                          Fraction(2) ** (f_in + int(f_w[k])))))(want[..., k])
            assert np.array_equal(y[..., k].astype(np.int64), ref.astype(np.int64)), k


def test_per_channel_conv_reduces_to_the_per_layer_one():
    """Equal formats in every channel give the per-layer result; in general channel k equals the
    per-layer convolution run with f_w[k] (the per-layer function is pinned above)."""
    rng = np.random.default_rng(77)
    x = rng.integers(-128, 128, (2, 6, 7, 8)).astype(np.int8)
    w = rng.integers(-128, 128, (5, 3, 3, 8)).astype(np.int8)
    b = rng.integers(-5000, 5000, (5,)).astype(np.int32)
    y0, _ = orc.conv_q(x, w, b, 4, 7, 3, 1, 1, 1, True)
    y1, _ = orc.conv_q(x, w, b, 4, np.full(5, 7, np.int32), 3, 1, 1, 1, True)
    assert np.array_equal(y0, y1)
    f_w = np.array([3, 9, 7, 12, 5], np.int32)
    y, _ = orc.conv_q(x, w, b, 4, f_w, 3, 2, 1, 1, False)
    for k in range(5):
        yk, _ = orc.conv_q(x, w, b, 4, int(f_w[k]), 3, 2, 1, 1, False)
        assert np.array_equal(y[..., k], yk[..., k])


def test_per_channel_scale_moves_between_codes_and_format():
    """Doubling channel k's weight and bias codes while raising f_w[k] by one names the same real
    weights, so the output cannot change - a per-layer format cannot express this."""
    rng = np.random.default_rng(78)
    x = rng.integers(-128, 128, (1, 5, 5, 4)).astype(np.int8)
    w = rng.integers(-60, 61, (3, 3, 3, 4)).astype(np.int8)
    b = rng.integers(-3000, 3000, (3,)).astype(np.int32)
    f_w = np.array([6, 6, 6], np.int32)
    y0, _ = orc.conv_q(x, w, b, 4, f_w, 2, 1, 1, 1, True)
    w2, b2, f2 = w.copy(), b.copy(), f_w.copy()
    w2[1] *= 2; b2[1] *= 2; f2[1] += 1
    y1, _ = orc.conv_q(x, w2, b2, 4, f2, 2, 1, 1, 1, True)
    assert np.array_equal(y0, y1)


def test_absmax_per_channel():
    a = np.array([[[1, -9, 0], [4, 2, -3]], [[-7, 8, 0], [2, 2, 2]]], np.int32)
    assert orc.absmax_i32_channels(a).tolist() == [7, 9, 3]
    assert orc.absmax_i32_channels(a, relu=True).tolist() == [4, 8, 2]
    rng = np.random.default_rng(5)
    r = rng.integers(-2 ** 31, 2 ** 31, (50, 7)).astype(np.int32)
    assert orc.absmax_i32_channels(r).tolist() == [orc.absmax_i32(r[:, k]) for k in range(7)]


# --------------------------------------------------------------------------- #
# Algorithm 1: threshold search on a histogram of magnitudes
# --------------------------------------------------------------------------- #

def test_histogram_of_magnitudes():
    rng = np.random.default_rng(41)
    for hi, relu in [(100, False), (5000, True), (2 ** 20, False), (2 ** 31 - 1, True)]:
        x = rng.integers(-hi, hi + 1, 3000).astype(np.int32)
        counts, j, m = orc.hist_i32(x, relu=relu)
        a = [max(int(v), 0) if relu else abs(int(v)) for v in x]
        assert m == max(a)
        assert (m >> j) < orc.NBINS and (j == 0 or (m >> (j - 1)) >= orc.NBINS)     # the smallest such shift
        want = [0] * ((m >> j) + 1)
        for v in a:
            want[v >> j] += 1
        assert counts.tolist() == want and int(counts.sum()) == len(x)
    counts, j, m = orc.hist_i32(np.zeros(7, np.int32))
    assert counts.tolist() == [7] and j == 0 and m == 0


def _interp_by_definition(x, xp, fp):
    """Piecewise-linear interpolation written out (xp increasing, x inside [xp[0], xp[-1]])."""
    out = []
    for v in x:
        k = max(t for t in range(len(xp)) if xp[t] <= v)
        if k == len(xp) - 1 or xp[k] == v:
            out.append(fp[k])
        else:
            out.append(fp[k] + (fp[k + 1] - fp[k]) * (v - xp[k]) / (xp[k + 1] - xp[k]))
    return out


def _threshold_by_steps(counts, j, m):
    """Algorithm 1 step by step in plain Python floats, with the readings listed in the oracle."""
    nb, total = len(counts), float(sum(counts))
    cdf, acc = [], 0.0
    for c in counts:
        acc += c / total
        cdf.append(acc)
    codes = [k / 127.0 for k in range(128)]
    best, gamma = float("inf"), m
    for i in range(129, nb + 1):
        r = cdf[:i - 1] + [1.0] * (nb - i + 1)
        grid = [t / (i - 1) for t in range(i)]
        r_interp = _interp_by_definition(codes, grid, r[:i])
        q = _interp_by_definition(grid, codes, r_interp) + r[i:]
        d = sum(abs(a - b) for a, b in zip(cdf, q))
        if best > d:
            best, gamma = d, min(i * 2 ** j - 1, m)
    return gamma, (0.0 if best == float("inf") else best)


def test_threshold_search_follows_the_algorithm_step_by_step():
    rng = np.random.default_rng(42)
    for scale, n, top in [(40.0, 4000, 170), (25.0, 3000, 260), (300.0, 5000, 2500)]:
        x = np.minimum(np.abs(rng.standard_normal(n) * scale), top).astype(np.int32)
        x[0] = top
        counts, j, m = orc.hist_i32(x)
        gamma, delta = orc.threshold_search(counts, j, m)
        g2, d2 = _threshold_by_steps([int(c) for c in counts], j, m)
        assert gamma == g2 and abs(delta - d2) <= 1e-9 * max(1.0, d2)


def test_threshold_search_hand_worked_histograms():
    """Three histograms whose search result is derived on paper (bin width 1, A elements per low bin, one element in
    the last bin).  With levels k/127 and the kept bins t/(i-1) on [0, 1], the requantized curve q differs from the
    data's distribution function only where a grid point falls strictly between two levels that hold different values.

    (a) 130 bins, A in bin 0: c = A/(A+1).  Keeping all 130 bins, the only such point is t = 128
        (128/129 - 126/127 = 2/(129*127), i.e. 2/129 of the way from level 126 to level 127): delta = (1-c) * 2/129.
        Clipping to 129 bins costs (1-c) at the bin that receives the clipped mass alone.  So gamma = max = 129.
    (b) 256 bins, A in bin 0: points t = 253 and 254 lie 1/255 and 128/255 of the way: delta = (1-c) * 129/255, again
        less than the (1-c) per clipped bin of any smaller candidate.  gamma = 255.
    (c) 2048 bins, A in bins 0 and 1 each: c0 = A/(2A+1), c1 = 2A/(2A+1).  Keeping 129 bins, level k lies between grid
        points k and k+1, so q follows the data except at t = 1 ((c1-c0)/128 short of c1) and t = 127 ((1-c1)/128 above
        c1); bin 128 and the 1918 clipped bins below the last one are off by (1-c1) each:
        delta = (c1-c0)/128 + (1-c1) * (1919 + 1/128).  Every larger candidate i pays at least
        (c1-c0) * (1 - 127/(i-1)) >= (c1-c0) * 2/129 at t = 1, which is more for large A.  gamma = 129 - 1 = 128."""
    A = 1000
    c = A / (A + 1.0)
    for nb, want_delta in [(130, (1 - c) * 2 / 129), (256, (1 - c) * 129 / 255)]:
        counts = np.zeros(nb, np.uint64); counts[0] = A; counts[-1] = 1
        gamma, delta = orc.threshold_search(counts, 0, nb - 1)
        assert gamma == nb - 1 and abs(delta - want_delta) <= 1e-9 * want_delta, (nb, gamma, delta)
    A = 10 ** 6                        # (c) needs 1919 / (2A+1) < (c1-c0) * (2/129 - 1/128), i.e. A > 249 000
    counts = np.zeros(2048, np.uint64); counts[0] = A; counts[1] = A; counts[-1] = 1
    c0, c1 = A / (2 * A + 1.0), 2 * A / (2 * A + 1.0)
    gamma, delta = orc.threshold_search(counts, 0, 2047)
    want = (c1 - c0) / 128 + (1 - c1) * (1919 + 1 / 128)
    assert gamma == 128 and abs(delta - want) <= 1e-9 * want, (gamma, delta, want)
    # the same three through the histogram front end (bin width 2: thresholds double, measures stay)
    x = np.concatenate([np.zeros(A, np.int32), np.ones(A, np.int32) * 2, np.array([4094], np.int32)])
    cnt, j, m = orc.hist_i32(x)
    assert j == 1 and m == 4094 and orc.threshold_search(cnt, j, m)[0] == 129 * 2 - 1


def test_threshold_search_properties():
    rng = np.random.default_rng(43)
    # too few bins to clip anything (the loop starts at 2^(n-1) + 1 = 129 bin edges): the maximum stays
    x = rng.integers(0, 100, 1000).astype(np.int32)
    counts, j, m = orc.hist_i32(x)
    assert orc.threshold_search(counts, j, m) == (m, 0.0)
    # an evenly filled range is not clipped (at most the partly filled last bin goes)
    x = rng.integers(0, 100000, 300000).astype(np.int32)
    counts, j, m = orc.hist_i32(x)
    assert m - 2 * 2 ** j < orc.threshold_search(counts, j, m)[0] <= m
    # one far outlier is clipped away, down to the smallest candidate, which still covers the bulk
    x = np.abs(rng.standard_normal(100000) * 3000).astype(np.int32)
    bulk = int(x.max())
    x[0] = 2_000_000
    counts, j, m = orc.hist_i32(x)
    gamma, delta = orc.threshold_search(counts, j, m)
    assert gamma == 129 * 2 ** j - 1 and bulk <= gamma < m and delta > 0
    # doubling every value doubles the bin width and nothing else
    c2, j2, m2 = orc.hist_i32(x * 2)
    assert j2 == j + 1 and np.array_equal(c2, counts)
    assert orc.threshold_search(c2, j2, m2)[0] == min(129 * 2 ** j2 - 1, m2)
    # all zeros
    assert orc.threshold_search(np.array([5], np.uint64), 0, 0) == (0, 0.0)


# --------------------------------------------------------------------------- #
# Preprocessing: an affine layer behind a convolution folded into its weights (Sec. 3)
# --------------------------------------------------------------------------- #

def test_fold_scale_is_the_affine_layer_applied_to_the_convolution():
    """z = scale[k] * (sum_j w[k][j] x[j] + b[k]) + shift[k] must equal the convolution with the folded weights:
    checked in double precision on random data (the folded float32 values are within half an ulp of the exact
    products), exactly for power-of-two scales, and row by row (the scale belongs to the OUTPUT channel)."""
    rng = np.random.default_rng(77)
    K, R, C = 6, 3, 5
    w = rng.standard_normal((K, R, R, C)).astype(np.float32)
    b = rng.standard_normal(K).astype(np.float32)
    scale = (rng.random(K) + 0.5).astype(np.float32)
    shift = (rng.standard_normal(K) * 0.1).astype(np.float32)
    w2, b2 = orc.fold_scale(w, b, scale, shift)
    x = rng.standard_normal((40, R * R * C))
    y = x @ w.reshape(K, -1).astype(np.float64).T + b.astype(np.float64)
    z = y * scale.astype(np.float64) + shift.astype(np.float64)
    z2 = x @ w2.reshape(K, -1).astype(np.float64).T + b2.astype(np.float64)
    assert np.abs(z - z2).max() <= 1e-6 * np.abs(x).sum(axis=1).max()
    # half-ulp bound element by element, against the exact rational product
    for k, i in [(0, 0), (3, 17), (5, 44)]:
        exact = Fraction(float(w.reshape(K, -1)[k, i])) * Fraction(float(scale[k]))
        got = Fraction(float(w2.reshape(K, -1)[k, i]))
        assert abs(got - exact) <= abs(exact) * Fraction(1, 2 ** 24)
    exact_b = Fraction(float(np.float32(b[2]) * np.float32(scale[2]))) + Fraction(float(shift[2]))     # product rounded first
    assert abs(Fraction(float(b2[2])) - exact_b) <= abs(exact_b) * Fraction(1, 2 ** 24)
    # powers of two: exact
    p2 = np.array([0.5, 2.0, 1.0, 4.0, 0.25, 8.0], np.float32)
    w3, b3 = orc.fold_scale(w, b, p2, None)
    assert np.array_equal(w3, w * p2[:, None, None, None]) and np.array_equal(b3, b * p2)
    # the scale of row k touches row k only; no bias and no shift give a zero bias
    one_hot = np.ones(K, np.float32); one_hot[4] = 3.0
    w4, b4 = orc.fold_scale(w, None, one_hot, None)
    assert np.array_equal(w4[:4], w[:4]) and np.array_equal(w4[5], w[5]) and not np.array_equal(w4[4], w[4])
    assert np.array_equal(b4, np.zeros(K, np.float32))


def test_conv_q_add_lazy_is_one_rounding_of_the_exact_sum():
    """The single-rounding join against exact rationals: value = acc * 2^-(f_in+f_w) + other * 2^-f_other, rounded once
    (nearest, ties to even) to f_out and clamped; where the convolution's own format loses nothing it must coincide with
    the two-rounding form (Eq. 6 then Eq. 10), and on a constructed case it must differ from it."""
    from fractions import Fraction
    rng = np.random.default_rng(404)
    N, H, W, C, K = 1, 3, 4, 8, 5
    x = rng.integers(-128, 128, (N, H, W, C)).astype(np.int8)
    w = rng.integers(-128, 128, (K, 1, 1, C)).astype(np.int8)
    b = rng.integers(-2000, 2000, K).astype(np.int32)
    other = rng.integers(-128, 128, (N, H, W, K)).astype(np.int8)
    for f_in, f_w, f_other, f_out, relu in [(4, 7, 5, 3, False), (4, 7, 5, 3, True), (3, 6, 9, 2, False), (5, 5, -2, -4, False),
                                            (6, 8, 4, 14, False), (2, 2, 4, 4, True)]:
        y = orc.conv_q_add_lazy(x, w, b, other, f_in, f_w, f_other, f_out, relu=relu)
        for idx in np.ndindex(N, H, W, K):
            n, p, q, k = idx
            acc = orc.conv_acc_at(x, w, b, 1, 0, 1, n, p, q, k)
            val = Fraction(acc, 1) / Fraction(2) ** (f_in + f_w) + Fraction(int(other[idx])) / Fraction(2) ** f_other
            if relu:
                val = max(val, Fraction(0))
            scaled = val * Fraction(2) ** f_out
            lo = scaled.numerator // scaled.denominator
            frac = scaled - lo
            r = lo + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and lo % 2) else 0)
            assert y[idx] == max(-127, min(127, r)), (idx, acc, int(other[idx]))
    # a convolution format as fine as the accumulator: nothing is lost by the first rounding, both forms agree
    xs = rng.integers(-3, 4, (1, 2, 2, 4)).astype(np.int8)
    ws = rng.integers(-3, 4, (3, 1, 1, 4)).astype(np.int8)
    os_ = rng.integers(-100, 100, (1, 2, 2, 3)).astype(np.int8)
    mid, _ = orc.conv_q(xs, ws, None, 2, 3, 5)
    two, _ = orc.eltwise_q(mid, 5, os_, 4, 3, False)
    assert np.array_equal(orc.conv_q_add_lazy(xs, ws, None, os_, 2, 3, 4, 3), two)
    # acc = 3 at scale 2^-2 (0.75), other = 1 at 2^0: two roundings give rne(rne(0.75) + 1) = 2, one rounding rne(1.75) = 2;
    # acc = 2 (0.5): rne(0.5) = 0 -> 0 + 1 = 1, but one rounding of 1.5 gives 2
    one = np.ones((1, 1, 1, 1), np.int8)
    for a_, want_two, want_one in [(3, 2, 2), (2, 1, 2), (6, 3, 2), (-2, 1, 0)]:
        xa = np.full((1, 1, 1, 1), a_, np.int8)
        mid, _ = orc.conv_q(xa, one, None, 1, 1, 0)
        two, _ = orc.eltwise_q(mid, 0, one, 0, 0, False)
        assert int(two[0, 0, 0, 0]) == want_two
        assert int(orc.conv_q_add_lazy(xa, one, None, one, 1, 1, 0, 0)[0, 0, 0, 0]) == want_one
    with pytest.raises(ValueError):
        orc.conv_q_add_lazy(x, w, b, other, 1, 1, 5, 0)          # second operand finer than the accumulator
