"""numpy front end of the CPU oracle (``dfq_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py``.  The GPU package never imports it and it never
imports the GPU package.  All arithmetic lives in the C file; this module only
marshals numpy arrays (NHWC activations, [K][R][S][C/groups] weights).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dfq_oracle.c")
_LIB = os.path.join(_HERE, "libdfq_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 and OpenMP (across output elements only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c99",
                               "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None

_i8p = C.POINTER(C.c_int8)
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_beta_max.restype = C.c_int64
        L.orc_beta_max.argtypes = [C.c_int, C.c_int]
        L.orc_mac_acc_bits.restype = C.c_int
        L.orc_mac_acc_bits.argtypes = [C.c_int64] * 5
        L.orc_mac_max_len.restype = C.c_int64
        L.orc_mac_max_len.argtypes = [C.c_int] + [C.c_int64] * 4
        L.orc_add_acc_bits.restype = C.c_int
        L.orc_add_acc_bits.argtypes = [C.c_int64] * 3
        L.orc_add_max_len.restype = C.c_int64
        L.orc_add_max_len.argtypes = [C.c_int, C.c_int64, C.c_int64]
        L.orc_rne_shift.restype = C.c_int64
        L.orc_rne_shift.argtypes = [C.c_int64, C.c_int]
        L.orc_requant8.restype = C.c_int
        L.orc_requant8.argtypes = [C.c_int64, C.c_int]
        L.orc_quantize.restype = None
        L.orc_quantize.argtypes = [_f32p, _i8p, C.c_size_t, C.c_int]
        L.orc_quantize_i32.restype = None
        L.orc_quantize_i32.argtypes = [_f32p, _i32p, C.c_size_t, C.c_int]
        L.orc_dequantize.restype = None
        L.orc_dequantize.argtypes = [_i8p, _f32p, C.c_size_t, C.c_int]
        L.orc_conv_acc_at.restype = C.c_int64
        L.orc_conv_acc_at.argtypes = [_i8p, _i8p, _i32p] + [C.c_int] * 14
        L.orc_conv_q.restype = C.c_int
        L.orc_conv_q.argtypes = [_i8p, _i8p, _i32p, _i8p, _i32p] + [C.c_int] * 15
        L.orc_conv_q_pc.restype = C.c_int
        L.orc_conv_q_pc.argtypes = [_i8p, _i8p, _i32p, _i8p, _i32p] + [C.c_int] * 12 + [_i32p, C.c_int, C.c_int]
        L.orc_absmax_i32_channels.restype = None
        L.orc_absmax_i32_channels.argtypes = [_i32p, C.c_size_t, C.c_int, C.c_int, C.POINTER(C.c_int64)]
        L.orc_add_lazy.restype = C.c_int
        L.orc_add_lazy.argtypes = [_i32p, _i8p, _i8p, C.c_size_t, C.c_int, C.c_int, C.c_int]
        L.orc_requant_i32.restype = None
        L.orc_requant_i32.argtypes = [_i32p, _i8p, C.c_size_t, C.c_int, C.c_int]
        L.orc_eltwise_q.restype = C.c_int
        L.orc_eltwise_q.argtypes = [_i8p, C.c_int, _i8p, C.c_int, _i8p, C.c_int, _i32p, C.c_size_t, C.c_int]
        L.orc_concat_q.restype = C.c_int
        L.orc_concat_q.argtypes = [C.c_int, C.POINTER(_i8p), C.POINTER(C.c_int), C.POINTER(C.c_int),
                                   _i8p, C.c_int, C.c_size_t]
        L.orc_pool_q.restype = C.c_int
        L.orc_pool_q.argtypes = [_i8p, _i8p] + [C.c_int] * 10
        L.orc_absmax_f32.restype = C.c_float
        L.orc_absmax_f32.argtypes = [_f32p, C.c_size_t]
        L.orc_absmax_i32.restype = C.c_int64
        L.orc_absmax_i32.argtypes = [_i32p, C.c_size_t, C.c_int]
        L.orc_frac_from_absmax_f32.restype = C.c_int
        L.orc_frac_from_absmax_f32.argtypes = [C.c_float]
        L.orc_frac_from_absmax_i32.restype = C.c_int
        L.orc_frac_from_absmax_i32.argtypes = [C.c_int64, C.c_int]
        L.orc_fold_scale.restype = None
        L.orc_fold_scale.argtypes = [_f32p, _f32p, C.c_size_t, C.c_size_t, _f32p, _f32p, _f32p, _f32p]
        L.orc_num_threads.restype = C.c_int
        L.orc_num_threads.argtypes = []
        _lib = L
    return _lib


def _c(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a, ptype):
    return None if a is None else a.ctypes.data_as(ptype)


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ---- closed forms ---------------------------------------------------------- #
def beta_max(n, p): return int(lib().orc_beta_max(n, p))
def mac_acc_bits(N, bx, ex=0, by=None, ey=0): return int(lib().orc_mac_acc_bits(N, bx, ex, bx if by is None else by, ey))
def mac_max_len(q, bx, ex=0, by=None, ey=0): return int(lib().orc_mac_max_len(q, bx, ex, bx if by is None else by, ey))
def add_acc_bits(N, bx, ex=0): return int(lib().orc_add_acc_bits(N, bx, ex))
def add_max_len(q, bx, ex=0): return int(lib().orc_add_max_len(q, bx, ex))
def rne_shift(v, s): return int(lib().orc_rne_shift(int(v), int(s)))
def requant8(v, s): return int(lib().orc_requant8(int(v), int(s)))


# ---- conversions ------------------------------------------------------------ #
def quantize(x: np.ndarray, f: int) -> np.ndarray:
    x = _c(x, np.float32)
    q = np.empty(x.shape, np.int8)
    lib().orc_quantize(_p(x, _f32p), _p(q, _i8p), x.size, int(f))
    return q


def quantize_i32(x: np.ndarray, f: int) -> np.ndarray:
    x = _c(x, np.float32)
    q = np.empty(x.shape, np.int32)
    lib().orc_quantize_i32(_p(x, _f32p), _p(q, _i32p), x.size, int(f))
    return q


def dequantize(q: np.ndarray, f: int) -> np.ndarray:
    q = _c(q, np.int8)
    x = np.empty(q.shape, np.float32)
    lib().orc_dequantize(_p(q, _i8p), _p(x, _f32p), q.size, int(f))
    return x


# ---- layers ------------------------------------------------------------------ #
def conv_out_hw(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def conv_q(x, w, b, f_in, f_w, f_out, stride=1, pad=0, groups=1, relu=False,
           want_y=True, want_acc=False):
    """Returns (y, acc): y int8 [N,P,Q,K] at f_out (or None), acc int32 [N,P,Q,K]
    including bias, before ReLU (or None).  Raises if an accumulator overflowed int32.
    f_w: one fractional length for the layer, or a sequence of K (one per output channel;
    b[k] is then at f_in + f_w[k])."""
    x = _c(x, np.int8); w = _c(w, np.int8)
    b = None if b is None else _c(b, np.int32)
    N, H, W, Cc = x.shape
    K, R, S, Cg = w.shape
    assert Cg * groups == Cc, "weight shape does not match C/groups"
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    y = np.empty((N, P, Q, K), np.int8) if want_y else None
    acc = np.empty((N, P, Q, K), np.int32) if want_acc else None
    if np.ndim(f_w) == 0:
        rc = lib().orc_conv_q(_p(x, _i8p), _p(w, _i8p), _p(b, _i32p), _p(y, _i8p), _p(acc, _i32p),
                              N, H, W, Cc, K, R, S, stride, pad, groups, K,
                              int(f_in), int(f_w), int(f_out), int(bool(relu)))
    else:
        fw = _c(f_w, np.int32)
        assert fw.shape == (K,), "one weight format per output channel"
        rc = lib().orc_conv_q_pc(_p(x, _i8p), _p(w, _i8p), _p(b, _i32p), _p(y, _i8p), _p(acc, _i32p),
                                 N, H, W, Cc, K, R, S, stride, pad, groups, K,
                                 int(f_in), _p(fw, _i32p), int(f_out), int(bool(relu)))
    if rc < 0:
        raise ValueError("oracle conv_q: bad shape")
    if rc > 0:
        raise OverflowError("oracle conv_q: accumulator exceeds int32 (Eq. 8/9 precondition)")
    return y, acc


def conv_acc_at(x, w, b, stride, pad, groups, n, p, q, k) -> int:
    x = _c(x, np.int8); w = _c(w, np.int8)
    b = None if b is None else _c(b, np.int32)
    N, H, W, Cc = x.shape
    K, R, S, Cg = w.shape
    return int(lib().orc_conv_acc_at(_p(x, _i8p), _p(w, _i8p), _p(b, _i32p), N, H, W, Cc, K, R, S,
                                     stride, pad, groups, n, p, q, k))


def requant_i32(acc, shift, relu=False):
    """int32 accumulators -> int8 codes: ReLU, rounding shift, clamp."""
    acc = _c(acc, np.int32)
    y = np.empty(acc.shape, np.int8)
    lib().orc_requant_i32(_p(acc, _i32p), _p(y, _i8p), acc.size, int(shift), int(bool(relu)))
    return y


def conv_q_add_lazy(x, w, b, other, f_in, f_w, f_other, f_out, stride=1, pad=0, groups=1, relu=False):
    """Convolution + element-wise add with a single rounding: the convolution's accumulator (at f_in + f_w, never
    rounded to a format of its own) plus `other` (int8 [N,P,Q,K] at f_other <= f_in + f_w, at most 22 bits coarser)
    brought to the accumulator's scale, ReLU on the sum if asked, one rounding shift to f_out."""
    _, acc = conv_q(x, w, b, f_in, f_w, 0, stride, pad, groups, False, want_y=False, want_acc=True)
    other = _c(other, np.int8)
    assert other.shape == acc.shape
    y = np.empty(acc.shape, np.int8)
    rc = lib().orc_add_lazy(_p(acc, _i32p), _p(other, _i8p), _p(y, _i8p), acc.size, int(f_in + f_w - f_other),
                            int(f_in + f_w - f_out), int(bool(relu)))
    if rc:
        raise ValueError("oracle conv_q_add_lazy: the second operand must be 0..22 bits coarser than the accumulator")
    return y


def eltwise_q(a, f_a, b, f_b, f_y, relu=False, want_y=True, want_acc=False):
    a = _c(a, np.int8); b = _c(b, np.int8)
    assert a.shape == b.shape
    y = np.empty(a.shape, np.int8) if want_y else None
    acc = np.empty(a.shape, np.int32) if want_acc else None
    rc = lib().orc_eltwise_q(_p(a, _i8p), int(f_a), _p(b, _i8p), int(f_b), _p(y, _i8p), int(f_y),
                             _p(acc, _i32p), a.size, int(bool(relu)))
    if rc:
        raise ValueError("oracle eltwise_q: formats too far apart")
    return y, acc


def concat_q(xs, fs, f_y):
    xs = [_c(x, np.int8) for x in xs]
    lead = xs[0].shape[:-1]
    assert all(x.shape[:-1] == lead for x in xs)
    Cs = [x.shape[-1] for x in xs]
    pixels = int(np.prod(lead))
    y = np.empty(lead + (sum(Cs),), np.int8)
    ptrs = (_i8p * len(xs))(*[_p(x, _i8p) for x in xs])
    rc = lib().orc_concat_q(len(xs), ptrs, (C.c_int * len(xs))(*Cs), (C.c_int * len(xs))(*[int(f) for f in fs]),
                            _p(y, _i8p), int(f_y), pixels)
    if rc:
        raise ValueError("oracle concat_q: bad arguments")
    return y


def pool_q(x, mode, k, stride, pad, f_in, f_out):
    """mode: 'max' or 'avg'."""
    x = _c(x, np.int8)
    N, H, W, Cc = x.shape
    P, Q = conv_out_hw(H, W, k, k, stride, pad)
    y = np.empty((N, P, Q, Cc), np.int8)
    rc = lib().orc_pool_q(_p(x, _i8p), _p(y, _i8p), {"max": 0, "avg": 1}[mode], N, H, W, Cc,
                          k, stride, pad, int(f_in), int(f_out))
    if rc:
        raise ValueError("oracle pool_q: bad arguments")
    return y


def fold_scale(w, b, scale, shift):
    """A per-channel affine layer behind a convolution folded into its float weights and bias:
    (w * scale[k], b * scale + shift), float32."""
    w = _c(w, np.float32); scale = _c(scale, np.float32)
    rows = w.shape[0]
    b = None if b is None else _c(b, np.float32)
    shift = None if shift is None else _c(shift, np.float32)
    w_out = np.empty_like(w)
    b_out = np.empty(rows, np.float32)
    lib().orc_fold_scale(_p(w, _f32p), _p(b, _f32p), rows, w.size // max(rows, 1), _p(scale, _f32p), _p(shift, _f32p),
                         _p(w_out, _f32p), _p(b_out, _f32p))
    return w_out, b_out


# ---- calibration building blocks ---------------------------------------------- #
def absmax_f32(x) -> float:
    x = _c(x, np.float32)
    return float(lib().orc_absmax_f32(_p(x, _f32p), x.size))


def absmax_i32(x, relu=False) -> int:
    x = _c(x, np.int32)
    return int(lib().orc_absmax_i32(_p(x, _i32p), x.size, int(bool(relu))))


def absmax_i32_channels(x, relu=False) -> np.ndarray:
    """Per-channel maximum of |x| over all leading axes of an [..., K] int32 array (int64 [K])."""
    x = _c(x, np.int32)
    K = x.shape[-1]
    out = np.zeros(K, np.int64)
    lib().orc_absmax_i32_channels(_p(x, _i32p), x.size // K, K, int(bool(relu)), out.ctypes.data_as(C.POINTER(C.c_int64)))
    return out


def frac_from_absmax_f32(gamma: float) -> int:
    f = int(lib().orc_frac_from_absmax_f32(float(gamma)))
    if f == -1000:
        raise ValueError("threshold must be finite and non-negative")
    return f


def frac_from_absmax_i32(m: int, acc_frac: int) -> int:
    f = int(lib().orc_frac_from_absmax_i32(int(m), int(acc_frac)))
    if f == -1000:
        raise ValueError("threshold must be non-negative")
    return f


# ---- Algorithm 1: threshold search on a histogram of magnitudes ------------------ #
# Readings taken where the algorithm leaves things open (each is restated in the design notes):
#   x            the layer's 32-bit accumulators after the ReLU (the tensor whose threshold is sought);
#   hist         at most NBINS = 2048 bins of power-of-two width 2^j over the integers |x|,
#                j the smallest shift with (max|x| >> j) < NBINS; bin_edges[i] = i * 2^j;
#   fpspace      the non-negative codes of the 8-bit format scaled to [0, 1]: k / 127, k = 0..127;
#   measure      the area between the two distribution functions, sum |cdf - q| over the bins;
#   gamma        the largest integer below bin_edges[i], but never above max|x|.
NBINS = 2048
N_CODES = 128


def hist_i32(x, relu=False):
    """Counts of |x| >> j per bin (uint64 [nb]), the shift j and max|x|; nb = (max|x| >> j) + 1 <= NBINS."""
    a = np.abs(np.maximum(_c(x, np.int32).astype(np.int64), 0) if relu else _c(x, np.int32).astype(np.int64)).ravel()
    m = int(a.max()) if a.size else 0
    j = 0
    while (m >> j) >= NBINS:
        j += 1
    nb = (m >> j) + 1
    counts = np.bincount(a >> j, minlength=nb).astype(np.uint64)
    return counts, j, m


def _clipped_and_requantized(cdf, i, levels):
    """Algorithm 1's two reference curves for the candidate that keeps the first i bins.
    r: the distribution function with all mass from bin i-1 on moved into bin i-1 (clipping at edge i).
    q: r as an 8-bit format over the clipped range [0, 1] can hold it - sampled at the format's levels,
    then brought back onto the bin grid by linear interpolation; beyond the kept bins q is r."""
    r = cdf.copy()
    r[i - 1:] = 1.0
    bins_on_unit_range = np.linspace(0.0, 1.0, i)
    r_at_levels = np.interp(levels, bins_on_unit_range, r[:i])
    q = r.copy()
    q[:i] = np.interp(bins_on_unit_range, levels, r_at_levels)
    return r, q


def threshold_search(counts, j, m):
    """Algorithm 1 on a histogram: returns (gamma, delta), gamma an integer threshold in the units of x.
    Candidates clip at bin edges i = 129 .. nb; a histogram with fewer bins than that is not clipped."""
    counts = np.asarray(counts, np.float64)
    nb = len(counts)
    total = counts.sum()
    if total == 0 or m == 0:
        return 0, 0.0
    cdf = np.cumsum(counts / total)
    levels = np.arange(N_CODES, dtype=np.float64) / float(N_CODES - 1)       # the non-negative 8-bit codes on [0, 1]
    gamma, delta = m, None                                                     # no candidate: nothing is clipped
    for i in range(N_CODES + 1, nb + 1):
        _, q = _clipped_and_requantized(cdf, i, levels)
        d = float(np.cumsum(np.abs(cdf - q))[-1])                              # the measure, summed in bin order
        if delta is None or delta > d:
            gamma, delta = min(i * (1 << j) - 1, m), d
    return int(gamma), float(0.0 if delta is None else delta)
