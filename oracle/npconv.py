"""Oracle of the multiply-accumulate on (n, p) dynamic floating-point codes (Sec. 2.2, Eq. 6-9).

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``): imported by ``tests/`` and by the ``cpu_baseline`` leg of
``bench.py`` alone.

Eq. 6: with x_i = alpha_x * beta_x_i and w_i = alpha_w * beta_w_i the output is
z = alpha_x * alpha_w * sum_i beta_x_i * beta_w_i, the sum of integer products taken without loss in an accumulator
wide enough for it (Eq. 8).  A convolution layer sums over the kernel window and the input channels of the output
channel's group; taps outside the image contribute nothing.  The bias is an integer at the accumulator's scale
alpha_x * alpha_w = 2^-(f_x + f_w) and is added to the sum; ReLU, where the layer has one, acts on that value.  The
result is then converted to the output format (n_y, p_y) at alpha_y = 2^-f_y as any real value is (``npfmt``:
nearest representable integer, ties to the even significand, saturation at +-beta_max), i.e. the accumulator value
times 2^-(f_x + f_w - f_y) is rounded ONCE.

Everything is exact integer arithmetic (numpy int64; the largest sums here stay below 2^40) up to the conversion, which
goes through float64 exactly (an integer below 2^53 times a power of two).
"""
from __future__ import annotations

import numpy as np

from . import npfmt as F


def decode_tensor(codes, n: int, p: int) -> np.ndarray:
    """Eq. 2 on every element: the integers beta (int64) of sign-and-magnitude codes."""
    table = np.array([F.decode(c, n, p) for c in range(1 << n)], np.int64)
    return table[np.asarray(codes).astype(np.int64)]


def out_hw(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def conv_sum(bx: np.ndarray, bw: np.ndarray, stride=1, pad=0, groups=1) -> np.ndarray:
    """The sum of Eq. 6 for every output: bx int64 [N,H,W,C], bw int64 [K,R,S,C/groups] -> int64 [N,P,Q,K]."""
    bx = np.asarray(bx, np.int64)
    bw = np.asarray(bw, np.int64)
    N, H, W, C = bx.shape
    K, R, S, Cg = bw.shape
    assert Cg * groups == C and K % groups == 0
    P, Q = out_hw(H, W, R, S, stride, pad)
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C), np.int64)
    xp[:, pad:pad + H, pad:pad + W, :] = bx
    Kg = K // groups
    acc = np.zeros((N, P, Q, K), np.int64)
    # Eq. 8: the whole sum of a window stays below R * S * Cg * max|beta_x| * max|beta_w|.  While that bound is below 2^53
    # every partial sum is an integer a double holds exactly, so the products of one tap may be summed by the library's
    # double-precision matrix product (a step of the definition, not a different algorithm); otherwise int64 throughout.
    bound = R * S * Cg * int(np.abs(bx).max(initial=0)) * int(np.abs(bw).max(initial=0))
    exact_in_double = bound < (1 << 53)
    for g in range(groups):
        for r in range(R):
            for s in range(S):
                win = xp[:, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride, g * Cg:(g + 1) * Cg]
                wt = bw[g * Kg:(g + 1) * Kg, r, s, :].T
                if exact_in_double:
                    acc[..., g * Kg:(g + 1) * Kg] += (win.astype(np.float64) @ wt.astype(np.float64)).astype(np.int64)
                else:
                    acc[..., g * Kg:(g + 1) * Kg] += win @ wt
    return acc


def convert(v, shift: int, fmt):
    """The conversion of Sec. 3 for integers v at one scale into the format fmt = (n, p) at a scale 2^shift times coarser:
    v * 2^-shift to the nearest representable integer, ties to the even significand, saturated; returns (codes, beta).
    |v| < 2^52, so the scaled value is exact in a double."""
    v = np.asarray(v, np.int64)
    assert np.abs(v).max(initial=0) < (1 << 52)
    beta = F.round_to_beta(np.ldexp(v.astype(np.float64), -int(shift)), *fmt)
    # magnitude -> code for the representable magnitudes (Eq. 2 inverted by enumerating the positive codes)
    enc = np.full(F.beta_max(*fmt) + 1, -1, np.int64)
    for c in range(1 << (fmt[0] - 1)):
        enc[F.decode(c, *fmt)] = c
    mag = np.abs(beta)
    assert (enc[mag] >= 0).all()
    codes = enc[mag] | np.where(beta < 0, 1 << (fmt[0] - 1), 0)
    return codes.astype(np.uint8 if fmt[0] <= 8 else np.uint16), beta


def conv_np(x_codes, fmt_x, w_codes, fmt_w, bias, shift: int, fmt_y, stride=1, pad=0, groups=1, relu=False):
    """x_codes uint8 [N,H,W,C] in format fmt_x = (n, p); w_codes [K,R,S,C/groups] in fmt_w; bias int [K] or None at the
    accumulator's scale; shift = f_x + f_w - f_y; returns (y_codes uint8 [N,P,Q,K] in fmt_y, beta_y int64, acc int64),
    acc being the sum plus bias before ReLU."""
    acc = conv_sum(decode_tensor(x_codes, *fmt_x), decode_tensor(w_codes, *fmt_w), stride, pad, groups)
    if bias is not None:
        acc = acc + np.asarray(bias, np.int64)[None, None, None, :]
    v = np.maximum(acc, 0) if relu else acc
    codes, beta = convert(v, shift, fmt_y)
    return codes, beta, acc


def eltwise_np(a_codes, fmt_a, f_a: int, b_codes, fmt_b, f_b: int, fmt_y, f_y: int, relu=False):
    """Eq. 10 on (n, p) codes with power-of-two scales: the two values alpha_a * beta_a and alpha_b * beta_b are brought to
    the finer of their scales by exact factors, summed without loss, ReLU acts on the sum if asked, and the sum is
    converted once to the output format at 2^-f_y (nearest representable integer, ties to the even significand,
    saturation).  Returns (codes, beta_y int64, sum int64 at the finer scale before ReLU)."""
    ba = decode_tensor(a_codes, *fmt_a)
    bb = decode_tensor(b_codes, *fmt_b)
    assert ba.shape == bb.shape
    F_ = max(int(f_a), int(f_b))
    t = ba * (1 << (F_ - int(f_a))) + bb * (1 << (F_ - int(f_b)))
    v = np.maximum(t, 0) if relu else t
    codes, beta = convert(v, F_ - int(f_y), fmt_y)
    return codes, beta, t


def pool_np(codes, fmt, mode: str, k: int, stride: int, pad: int = 0):
    """Pooling on (n, p) codes [N,H,W,C]; the result keeps the input's format and scale.
    "max": the largest value of the window's taps inside the image (Eq. 2 is monotone in the value, so the result is one
    of the input codes; -0 counts as 0 and comes out as +0).  "avg" (unpadded windows only): the exact mean of the k * k
    integers, converted to the format as any real value is.  The mean is a multiple of 1 / k^2 below 2^13; a tie of the
    format is a multiple of 1/2, so a mean that is not a tie is at least 1 / (2 k^2) away from one and the double
    quotient (error below 2^-39) rounds as the exact rational does, while exact ties are dyadic and exact in a double."""
    beta = decode_tensor(codes, *fmt)
    N, H, W, C = beta.shape
    P, Q = out_hw(H, W, k, k, stride, pad)
    if mode == "max":
        lowest = -F.beta_max(*fmt) - 1
        xp = np.full((N, H + 2 * pad, W + 2 * pad, C), lowest, np.int64)
        xp[:, pad:pad + H, pad:pad + W, :] = beta
        out = np.full((N, P, Q, C), lowest, np.int64)
        for r in range(k):
            for s in range(k):
                out = np.maximum(out, xp[:, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride, :])
        assert (out > lowest).all()
        return convert(out, 0, fmt)
    if mode != "avg" or pad != 0:
        raise ValueError("average pooling over unpadded windows, or max pooling")
    tot = np.zeros((N, P, Q, C), np.int64)
    for r in range(k):
        for s in range(k):
            tot += beta[:, r:r + stride * (P - 1) + 1:stride, s:s + stride * (Q - 1) + 1:stride, :]
    b = F.round_to_beta(tot.astype(np.float64) / float(k * k), *fmt)
    # encode through convert(): the rounded integers are representable, so this conversion changes nothing
    return convert(b, 0, fmt)


def conv_sum_at(bx, bw, bias, stride, pad, groups, n, p, q, k) -> int:
    """One output's accumulator (sum + bias) by plain loops over Python integers."""
    N, H, W, C = bx.shape
    K, R, S, Cg = bw.shape
    g = k // (K // groups)
    tot = 0 if bias is None else int(bias[k])
    for r in range(R):
        ih = p * stride - pad + r
        if ih < 0 or ih >= H:
            continue
        for s in range(S):
            iw = q * stride - pad + s
            if iw < 0 or iw >= W:
                continue
            xa = bx[n, ih, iw, g * Cg:(g + 1) * Cg]
            wa = bw[k, r, s, :]
            tot += sum(int(a) * int(b) for a, b in zip(xa.tolist(), wa.tolist()))
    return tot
