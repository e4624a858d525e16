"""ctypes binding of libdfq.so: one Python function per C entry point of include/dfq.h.

Argument marshalling only.  Tensors are torch CUDA tensors (PyTorch supplies device
memory and the current HIP stream); every arithmetic step runs inside the library's
kernels.  There is no fallback: if the shared library is missing the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdfq.so")

OK, EINVAL, ESHAPE, EFMT, EUNSUPPORTED, EDEVICE = range(6)
POOL_MAX, POOL_AVG = 0, 1
CONV_AUTO, CONV_DIRECT, CONV_MFMA, CONV_DEPTHWISE, CONV_SMALLC, CONV_POINTWISE, CONV_GROUPED = range(7)
CONV_VARIANT_NAMES = {CONV_AUTO: "auto", CONV_DIRECT: "direct", CONV_MFMA: "mfma",
                      CONV_DEPTHWISE: "depthwise", CONV_SMALLC: "smallc", CONV_POINTWISE: "pointwise",
                      CONV_GROUPED: "grouped"}

EXPORTS = [
    "dfq_status_string", "dfq_quantize", "dfq_quantize_i32", "dfq_dequantize", "dfq_quantize_np", "dfq_dequantize_np", "dfq_conv_q",
    "dfq_conv_q_variant", "dfq_conv_q_select", "dfq_conv_q_add", "dfq_conv_q_pc", "dfq_conv_q_pc_add", "dfq_absmax_i32_channels", "dfq_hist_i32", "dfq_threshold_search", "dfq_absmax_f32_rows", "dfq_quantize_rows", "dfq_quantize_i32_rows", "dfq_fold_scale_f32", "dfq_eltwise_q", "dfq_concat_q", "dfq_concat_q_into", "dfq_pool_q",
    "dfq_absmax_f32", "dfq_absmax_i32", "dfq_fmt_from_absmax_f32", "dfq_fmt_from_absmax_i32", "dfq_hist_shift", "dfq_fmt_from_absmax_i32_channels",
    "dfq_beta_max", "dfq_mac_acc_bits", "dfq_mac_max_len", "dfq_add_acc_bits", "dfq_add_max_len",
    "dfq_np_digits", "dfq_conv_np", "dfq_conv_np_variant", "dfq_np_frac_from_absmax_f32", "dfq_conv_q_add_lazy", "dfq_eltwise_np",
    "dfq_conv_np_absmax", "dfq_eltwise_np_absmax", "dfq_np_frac_from_absmax_u64", "dfq_pool_np", "dfq_stem_pack_x", "dfq_stem_pack_w", "dfq_conv_np_add",
    "dfq_conv_q_maxpool", "dfq_quantize_conv_q_maxpool", "dfq_conv_q_pc_maxpool", "dfq_quantize_conv_q_pc_maxpool", "dfq_quantize_conv_q",
]


class Fmt(C.Structure):
    """dfq_fmt: value = code * 2^-frac, bits must be 8."""
    _fields_ = [("bits", C.c_int32), ("frac", C.c_int32)]


def fmt(frac: int) -> Fmt:
    return Fmt(8, int(frac))


class DfqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib():
    """Loads libdfq.so (built by paper_1805_07941_amd.build); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1805_07941_amd.build` "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
    L.dfq_status_string.restype = C.c_char_p
    L.dfq_status_string.argtypes = [i32]
    L.dfq_quantize.argtypes = [vp, vp, sz, Fmt, vp]
    L.dfq_quantize_i32.argtypes = [vp, vp, sz, C.c_int32, vp]
    L.dfq_dequantize.argtypes = [vp, vp, sz, Fmt, vp]
    L.dfq_quantize_np.argtypes = [vp, vp, sz, i32, i32, i32, vp]
    L.dfq_dequantize_np.argtypes = [vp, vp, sz, i32, i32, i32, vp]
    conv_args = [vp, vp, vp, vp, vp] + [i32] * 11 + [Fmt, Fmt, Fmt, i32, vp]
    L.dfq_conv_q.argtypes = conv_args
    L.dfq_conv_q_variant.argtypes = [i32] + conv_args
    L.dfq_conv_q_pc.argtypes = [vp, vp, vp, vp, vp] + [i32] * 11 + [Fmt, vp, i32, i32, Fmt, i32, vp]
    L.dfq_conv_q_pc_add.argtypes = [vp, vp, vp, vp, vp] + [i32] * 12 + [Fmt, vp, i32, i32, Fmt, i32, Fmt, Fmt, i32, vp]
    L.dfq_absmax_i32_channels.argtypes = [vp, sz, i32, i32, vp, vp]
    L.dfq_hist_i32.argtypes = [vp, sz, i32, i32, vp, vp]
    L.dfq_threshold_search.argtypes = [vp, i32, i32, i64, C.POINTER(i64), C.POINTER(C.c_double)]
    L.dfq_absmax_f32_rows.argtypes = [vp, sz, sz, vp, vp]
    L.dfq_quantize_rows.argtypes = [vp, vp, sz, sz, vp, vp]
    L.dfq_quantize_i32_rows.argtypes = [vp, vp, sz, sz, vp, i32, vp]
    L.dfq_fold_scale_f32.argtypes = [vp, vp, sz, sz, vp, vp, vp, vp, vp]
    L.dfq_conv_q_select.argtypes = [i32] * 10
    L.dfq_conv_q_add.argtypes = [vp, vp, vp, vp, vp] + [i32] * 12 + [Fmt, Fmt, Fmt, i32, Fmt, Fmt, i32, vp]
    L.dfq_conv_q_add_lazy.argtypes = [vp, vp, vp, vp, vp] + [i32] * 12 + [Fmt, Fmt, Fmt, Fmt, i32, vp]
    L.dfq_conv_q_add_lazy.restype = i32
    L.dfq_conv_q_maxpool.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [Fmt, Fmt, Fmt, i32, i32, i32, i32, vp]
    L.dfq_conv_q_maxpool.restype = i32
    L.dfq_quantize_conv_q_maxpool.argtypes = L.dfq_conv_q_maxpool.argtypes
    L.dfq_quantize_conv_q_maxpool.restype = i32
    L.dfq_conv_q_pc_maxpool.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [Fmt, vp, i32, i32, Fmt, i32, i32, i32, i32, vp]
    L.dfq_conv_q_pc_maxpool.restype = i32
    L.dfq_quantize_conv_q_pc_maxpool.argtypes = L.dfq_conv_q_pc_maxpool.argtypes
    L.dfq_quantize_conv_q_pc_maxpool.restype = i32
    L.dfq_quantize_conv_q.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [Fmt, Fmt, Fmt, i32, vp]
    L.dfq_quantize_conv_q.restype = i32
    L.dfq_eltwise_q.argtypes = [vp, Fmt, vp, Fmt, vp, Fmt, vp, sz, i32, vp]
    L.dfq_concat_q.argtypes = [i32, C.POINTER(vp), C.POINTER(i32), C.POINTER(Fmt), vp, Fmt, sz, vp]
    L.dfq_concat_q_into.argtypes = [i32, C.POINTER(vp), C.POINTER(i32), C.POINTER(Fmt), vp, i32, Fmt, sz, vp]
    L.dfq_pool_q.argtypes = [vp, vp, i32] + [i32] * 7 + [Fmt, Fmt, vp]
    L.dfq_absmax_f32.argtypes = [vp, sz, vp, vp]
    L.dfq_absmax_i32.argtypes = [vp, sz, i32, vp, vp]
    L.dfq_fmt_from_absmax_f32.argtypes = [C.c_float, C.POINTER(Fmt)]
    L.dfq_fmt_from_absmax_i32.argtypes = [i64, C.c_int32, C.POINTER(Fmt)]
    L.dfq_fmt_from_absmax_i32_channels.argtypes = [vp, i32, C.c_int32, vp, C.POINTER(Fmt)]
    L.dfq_np_digits.argtypes = [vp, sz, i32, vp, vp, vp]
    L.dfq_conv_np.argtypes = [vp] * 8 + [i32] * 15 + [vp]
    L.dfq_conv_np_variant.argtypes = [i32] + [vp] * 8 + [i32] * 15 + [vp]
    L.dfq_eltwise_np.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, vp, i32, i32, sz, i32, vp]
    L.dfq_eltwise_np.restype = i32
    L.dfq_conv_np_add.argtypes = [vp] * 9 + [i32] * 18 + [vp]
    L.dfq_conv_np_add.restype = i32
    L.dfq_conv_np_absmax.argtypes = [vp] * 6 + [i32] * 11 + [vp]
    L.dfq_conv_np_absmax.restype = i32
    L.dfq_eltwise_np_absmax.argtypes = [vp, vp, i32, vp, vp, i32, vp, sz, i32, vp]
    L.dfq_eltwise_np_absmax.restype = i32
    L.dfq_np_frac_from_absmax_u64.argtypes = [C.c_uint64, i32, i32, i32, C.POINTER(i32)]
    L.dfq_np_frac_from_absmax_u64.restype = i32
    L.dfq_pool_np.argtypes = [vp] * 5 + [i32] * 9 + [vp]
    L.dfq_pool_np.restype = i32
    L.dfq_stem_pack_x.argtypes = [vp, vp] + [i32] * 7 + [vp]
    L.dfq_stem_pack_x.restype = i32
    L.dfq_stem_pack_w.argtypes = [vp, vp] + [i32] * 4 + [vp]
    L.dfq_stem_pack_w.restype = i32
    L.dfq_np_frac_from_absmax_f32.argtypes = [C.c_float, i32, i32, C.POINTER(C.c_int32)]
    for name in ("dfq_np_digits", "dfq_conv_np", "dfq_conv_np_variant", "dfq_np_frac_from_absmax_f32"):
        getattr(L, name).restype = i32
    L.dfq_hist_shift.argtypes = [i64]
    L.dfq_hist_shift.restype = i32
    for name in ("dfq_quantize", "dfq_quantize_i32", "dfq_dequantize", "dfq_conv_q", "dfq_conv_q_variant",
                 "dfq_conv_q_select", "dfq_conv_q_add", "dfq_eltwise_q", "dfq_concat_q", "dfq_concat_q_into", "dfq_pool_q", "dfq_absmax_f32",
                 "dfq_absmax_i32", "dfq_fmt_from_absmax_f32", "dfq_fmt_from_absmax_i32", "dfq_fmt_from_absmax_i32_channels",
                 "dfq_conv_q_pc", "dfq_conv_q_pc_add", "dfq_absmax_i32_channels", "dfq_absmax_f32_rows", "dfq_quantize_rows",
                 "dfq_quantize_i32_rows", "dfq_hist_i32", "dfq_threshold_search", "dfq_fold_scale_f32", "dfq_quantize_np",
                 "dfq_dequantize_np"):
        getattr(L, name).restype = i32
    L.dfq_beta_max.restype = i64
    L.dfq_beta_max.argtypes = [i32, i32]
    L.dfq_mac_acc_bits.restype = i32
    L.dfq_mac_acc_bits.argtypes = [i64] * 5
    L.dfq_mac_max_len.restype = i64
    L.dfq_mac_max_len.argtypes = [i32] + [i64] * 4
    L.dfq_add_acc_bits.restype = i32
    L.dfq_add_acc_bits.argtypes = [i64] * 3
    L.dfq_add_max_len.restype = i64
    L.dfq_add_max_len.argtypes = [i32, i64, i64]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().dfq_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise DfqError(status, where)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _dev(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of {dtype}")
    return t


# ---- conversions ------------------------------------------------------------------ #
def quantize(x: torch.Tensor, frac: int, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    _dev(x, torch.float32, "x")
    q = out if out is not None else torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _check(lib().dfq_quantize(_ptr(x), _ptr(q), x.numel(), fmt(frac), _stream(stream)), "dfq_quantize")
    return q


def quantize_i32(x: torch.Tensor, frac: int, stream=None) -> torch.Tensor:
    _dev(x, torch.float32, "x")
    q = torch.empty(x.shape, dtype=torch.int32, device=x.device)
    _check(lib().dfq_quantize_i32(_ptr(x), _ptr(q), x.numel(), int(frac), _stream(stream)), "dfq_quantize_i32")
    return q


def dequantize(q: torch.Tensor, frac: int, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    _dev(q, torch.int8, "q")
    x = out if out is not None else torch.empty(q.shape, dtype=torch.float32, device=q.device)
    _check(lib().dfq_dequantize(_ptr(q), _ptr(x), q.numel(), fmt(frac), _stream(stream)), "dfq_dequantize")
    return x


def quantize_np(x: torch.Tensor, nbits: int, p: int, frac: int, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """float32 -> (nbits, p) dynamic floating-point codes (Eq. 2), one per byte (uint8 tensor)."""
    _dev(x, torch.float32, "x")
    q = out if out is not None else torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    _check(lib().dfq_quantize_np(_ptr(x), _ptr(q), x.numel(), int(nbits), int(p), int(frac), _stream(stream)), "dfq_quantize_np")
    return q


def dequantize_np(q: torch.Tensor, nbits: int, p: int, frac: int, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    _dev(q, torch.uint8, "q")
    x = out if out is not None else torch.empty(q.shape, dtype=torch.float32, device=q.device)
    _check(lib().dfq_dequantize_np(_ptr(q), _ptr(x), q.numel(), int(nbits), int(p), int(frac), _stream(stream)), "dfq_dequantize_np")
    return x


def np_digits(codes: torch.Tensor, p: int, stream=None):
    """(8, p) codes (uint8) -> digit planes (hi, lo) of their integers beta = 64 * hi + lo (int8 tensors)."""
    _dev(codes, torch.uint8, "codes")
    hi = torch.empty(codes.shape, dtype=torch.int8, device=codes.device)
    lo = torch.empty_like(hi)
    _check(lib().dfq_np_digits(_ptr(codes), codes.numel(), int(p), _ptr(hi), _ptr(lo), _stream(stream)), "dfq_np_digits")
    return hi, lo


def conv_np(xh: torch.Tensor, xl: torch.Tensor, wh: torch.Tensor, wl: torch.Tensor, b: Optional[torch.Tensor],
            f_x: int, f_w: int, f_y: int, p_y: int, stride: int = 1, pad: int = 0, groups: int = 1, relu: bool = False,
            want_codes: bool = True, want_digits: bool = True, variant: int = CONV_AUTO, out=None, stream=None):
    """Convolution on (8, p >= 4) codes held as digit planes.  xh, xl [N,H,W,C] int8; wh, wl [K,R,S,C/groups] int8;
    b [K] int32 or None.  Returns (codes uint8 or None, yh, yl or None, None); `out` = (codes, yh, yl) supplies buffers."""
    for t, name in ((xh, "xh"), (xl, "xl"), (wh, "wh"), (wl, "wl")):
        _dev(t, torch.int8, name)
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = xh.shape
    K, R, S, Cg = wh.shape
    if Cg * groups != Cc or xl.shape != xh.shape or wl.shape != wh.shape:
        raise ValueError("operand shapes do not match")
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    if out is not None:
        y, yh, yl = out
    else:
        y = torch.empty((N, P, Q, K), dtype=torch.uint8, device=xh.device) if want_codes else None
        yh = torch.empty((N, P, Q, K), dtype=torch.int8, device=xh.device) if want_digits else None
        yl = torch.empty((N, P, Q, K), dtype=torch.int8, device=xh.device) if want_digits else None
    _check(lib().dfq_conv_np_variant(int(variant), _ptr(xh), _ptr(xl), _ptr(wh), _ptr(wl), _ptr(b), _ptr(y), _ptr(yh), _ptr(yl),
                                     N, H, W, Cc, K, R, S, int(stride), int(pad), int(groups), int(f_x), int(f_w), int(f_y), int(p_y),
                                     int(bool(relu)), _stream(stream)), "dfq_conv_np")
    return y, yh, yl


def eltwise_np(ah: torch.Tensor, al: torch.Tensor, f_a: int, bh: torch.Tensor, bl: torch.Tensor, f_b: int, f_y: int, p_y: int,
               relu: bool = False, want_codes: bool = True, want_digits: bool = True, stream=None):
    """Element-wise add of two (8, p >= 4) tensors held as digit planes (Eq. 10).  Returns (codes or None, yh, yl or None, None)."""
    for t, name in ((ah, "ah"), (al, "al"), (bh, "bh"), (bl, "bl")):
        _dev(t, torch.int8, name)
    if not (ah.shape == al.shape == bh.shape == bl.shape):
        raise ValueError("operand shapes do not match")
    y = torch.empty(ah.shape, dtype=torch.uint8, device=ah.device) if want_codes else None
    yh = torch.empty(ah.shape, dtype=torch.int8, device=ah.device) if want_digits else None
    yl = torch.empty(ah.shape, dtype=torch.int8, device=ah.device) if want_digits else None
    _check(lib().dfq_eltwise_np(_ptr(ah), _ptr(al), int(f_a), _ptr(bh), _ptr(bl), int(f_b), _ptr(y), _ptr(yh), _ptr(yl), int(f_y), int(p_y),
                                ah.numel(), int(bool(relu)), _stream(stream)), "dfq_eltwise_np")
    return y, yh, yl


def conv_np_add(xh, xl, wh, wl, b, oh, ol, f_x: int, f_w: int, f_mid: int, relu_mid: bool, f_other: int, f_y: int, p: int, relu_out: bool,
                stride: int = 1, pad: int = 0, groups: int = 1, out=None, stream=None):
    """Convolution on (8, p) digit planes with the element-wise add behind it taken in its epilogue (see dfq_conv_np_add).
    Returns (yh, yl); raises DfqError(EUNSUPPORTED) where the library has no fused kernel for the case."""
    for t, name in ((xh, "xh"), (xl, "xl"), (wh, "wh"), (wl, "wl"), (oh, "oh"), (ol, "ol")):
        _dev(t, torch.int8, name)
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = xh.shape
    K, R, S, Cg = wh.shape
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    if Cg * groups != Cc or xl.shape != xh.shape or wl.shape != wh.shape or tuple(oh.shape) != (N, P, Q, K) or ol.shape != oh.shape:
        raise ValueError("operand shapes do not match")
    yh, yl = out if out is not None else (torch.empty_like(oh), torch.empty_like(oh))
    _check(lib().dfq_conv_np_add(_ptr(xh), _ptr(xl), _ptr(wh), _ptr(wl), _ptr(b), _ptr(oh), _ptr(ol), _ptr(yh), _ptr(yl), N, H, W, Cc, K, R, S,
                                 int(stride), int(pad), int(groups), int(f_x), int(f_w), int(f_mid), int(bool(relu_mid)), int(f_other), int(f_y),
                                 int(p), int(bool(relu_out)), _stream(stream)), "dfq_conv_np_add")
    return yh, yl


def _read_u64(t: torch.Tensor) -> int:
    return int(t.cpu()[0])


def conv_np_absmax(xh, xl, wh, wl, b, stride: int = 1, pad: int = 0, groups: int = 1, relu: bool = False, stream=None) -> int:
    """Largest |sum + bias| of the layer (after ReLU if asked) as a Python integer at the accumulator's scale; synchronizes."""
    for t, name in ((xh, "xh"), (xl, "xl"), (wh, "wh"), (wl, "wl")):
        _dev(t, torch.int8, name)
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = xh.shape
    K, R, S, Cg = wh.shape
    if Cg * groups != Cc or xl.shape != xh.shape or wl.shape != wh.shape:
        raise ValueError("operand shapes do not match")
    out = torch.empty(1, dtype=torch.int64, device=xh.device)
    _check(lib().dfq_conv_np_absmax(_ptr(xh), _ptr(xl), _ptr(wh), _ptr(wl), _ptr(b), _ptr(out), N, H, W, Cc, K, R, S, int(stride), int(pad),
                                    int(groups), int(bool(relu)), _stream(stream)), "dfq_conv_np_absmax")
    return _read_u64(out)


def eltwise_np_absmax(ah, al, f_a: int, bh, bl, f_b: int, relu: bool = False, stream=None) -> int:
    for t, name in ((ah, "ah"), (al, "al"), (bh, "bh"), (bl, "bl")):
        _dev(t, torch.int8, name)
    if not (ah.shape == al.shape == bh.shape == bl.shape):
        raise ValueError("operand shapes do not match")
    out = torch.empty(1, dtype=torch.int64, device=ah.device)
    _check(lib().dfq_eltwise_np_absmax(_ptr(ah), _ptr(al), int(f_a), _ptr(bh), _ptr(bl), int(f_b), _ptr(out), ah.numel(), int(bool(relu)),
                                       _stream(stream)), "dfq_eltwise_np_absmax")
    return _read_u64(out)


def np_frac_from_absmax_u64(m: int, acc_frac: int, nbits: int, p: int) -> int:
    f = C.c_int32()
    _check(lib().dfq_np_frac_from_absmax_u64(int(m), int(acc_frac), int(nbits), int(p), C.byref(f)), "dfq_np_frac_from_absmax_u64")
    return int(f.value)


def pool_np(xh: torch.Tensor, xl: torch.Tensor, mode: str, k: int, stride: int, pad: int, p: int, want_codes: bool = True,
            want_digits: bool = True, out=None, stream=None):
    """Pooling on (8, p) digit planes [N,H,W,C]; mode "max" or "avg".  Returns (codes or None, yh, yl or None, None)."""
    _dev(xh, torch.int8, "xh")
    _dev(xl, torch.int8, "xl")
    if xh.shape != xl.shape:
        raise ValueError("operand shapes do not match")
    N, H, W, Cc = xh.shape
    P, Q = conv_out_hw(H, W, k, k, stride, pad)
    if out is not None:
        y, yh, yl = out
    else:
        y = torch.empty((N, P, Q, Cc), dtype=torch.uint8, device=xh.device) if want_codes else None
        yh = torch.empty((N, P, Q, Cc), dtype=torch.int8, device=xh.device) if want_digits else None
        yl = torch.empty((N, P, Q, Cc), dtype=torch.int8, device=xh.device) if want_digits else None
    _check(lib().dfq_pool_np(_ptr(xh), _ptr(xl), _ptr(y), _ptr(yh), _ptr(yl), {"max": POOL_MAX, "avg": POOL_AVG}[mode], N, H, W, Cc, int(k),
                             int(stride), int(pad), int(p), _stream(stream)), "dfq_pool_np")
    return y, yh, yl


def stem_pack_x(x: torch.Tensor, R: int, S: int, pad: int, out=None, stream=None) -> torch.Tensor:
    """One byte tensor [N,H,W,C <= 4] of a stride-2 first layer -> [N, P + 3, Q, 64] (see dfq_stem_pack_x)."""
    if not x.is_cuda or x.element_size() != 1 or not x.is_contiguous():
        raise ValueError("x must be a contiguous one-byte device tensor")
    N, H, W, Cc = x.shape
    P, Q = conv_out_hw(H, W, R, S, 2, pad)
    y = out if out is not None else torch.empty((N, P + 3, Q, 64), dtype=x.dtype, device=x.device)
    _check(lib().dfq_stem_pack_x(_ptr(x), _ptr(y), N, H, W, Cc, int(R), int(S), int(pad), _stream(stream)), "dfq_stem_pack_x")
    return y


def stem_pack_w(w: torch.Tensor, stream=None) -> torch.Tensor:
    """One byte tensor of weights [K,R,S,C <= 4] -> [K, 4, 1, 64] (see dfq_stem_pack_w)."""
    if not w.is_cuda or w.element_size() != 1 or not w.is_contiguous():
        raise ValueError("w must be a contiguous one-byte device tensor")
    K, R, S, Cc = w.shape
    y = torch.empty((K, 4, 1, 64), dtype=w.dtype, device=w.device)
    _check(lib().dfq_stem_pack_w(_ptr(w), _ptr(y), K, R, S, Cc, _stream(stream)), "dfq_stem_pack_w")
    return y


# ---- layers ---------------------------------------------------------------------- #
def conv_out_hw(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def conv_q(x: torch.Tensor, w: torch.Tensor, b: Optional[torch.Tensor], f_in: int, f_w: int, f_out: int,
           stride: int = 1, pad: int = 0, groups: int = 1, relu: bool = False,
           out: Optional[torch.Tensor] = None, ldy: Optional[int] = None,
           want_y: bool = True, want_acc: bool = False, acc_out: Optional[torch.Tensor] = None,
           variant: int = CONV_AUTO, stream=None):
    """x [N,H,W,C] int8, w [K,R,S,C/groups] int8, b [K] int32 or None.  Returns (y, acc).
    `out` may be a preallocated destination (with `ldy` bytes per pixel when it is a channel
    slice of a wider tensor)."""
    _dev(x, torch.int8, "x"); _dev(w, torch.int8, "w")
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = x.shape
    K, R, S, Cg = w.shape
    if Cg * groups != Cc:
        raise DfqError(ESHAPE, "conv_q (weight shape does not match C/groups)")
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    y = out
    if y is None and want_y:
        y = torch.empty((N, max(P, 0), max(Q, 0), K), dtype=torch.int8, device=x.device)
    acc = acc_out
    if acc is None and want_acc:
        acc = torch.empty((N, max(P, 0), max(Q, 0), K), dtype=torch.int32, device=x.device)
    st = lib().dfq_conv_q_variant(int(variant), _ptr(x), _ptr(w), _ptr(b), _ptr(y), _ptr(acc),
                                  N, H, W, Cc, K, R, S, stride, pad, groups, K if ldy is None else int(ldy),
                                  fmt(f_in), fmt(f_w), fmt(f_out), int(bool(relu)), _stream(stream))
    _check(st, "dfq_conv_q")
    return y, acc


def conv_q_pc(x: torch.Tensor, w: torch.Tensor, b: Optional[torch.Tensor], f_in: int, frac_w: torch.Tensor, f_out: int,
              stride: int = 1, pad: int = 0, groups: int = 1, relu: bool = False,
              out: Optional[torch.Tensor] = None, ldy: Optional[int] = None,
              want_y: bool = True, want_acc: bool = False, acc_out: Optional[torch.Tensor] = None,
              frac_w_range=None, stream=None):
    """conv_q with one weight format per output channel: frac_w is an int32 device tensor [K];
    b[k] is at f_in + frac_w[k].  frac_w_range = (lowest, highest) entry as the caller knows them; read
    back from the device (a synchronization) when not given.  Returns (y, acc)."""
    _dev(x, torch.int8, "x"); _dev(w, torch.int8, "w"); _dev(frac_w, torch.int32, "frac_w")
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = x.shape
    K, R, S, Cg = w.shape
    if Cg * groups != Cc:
        raise DfqError(ESHAPE, "conv_q_pc (weight shape does not match C/groups)")
    if tuple(frac_w.shape) != (K,):
        raise DfqError(ESHAPE, "conv_q_pc (one weight format per output channel)")
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    y = out
    if y is None and want_y:
        y = torch.empty((N, max(P, 0), max(Q, 0), K), dtype=torch.int8, device=x.device)
    acc = acc_out
    if acc is None and want_acc:
        acc = torch.empty((N, max(P, 0), max(Q, 0), K), dtype=torch.int32, device=x.device)
    if frac_w_range is None:
        fh = frac_w.cpu()
        frac_w_range = (int(fh.min()), int(fh.max()))
    st = lib().dfq_conv_q_pc(_ptr(x), _ptr(w), _ptr(b), _ptr(y), _ptr(acc), N, H, W, Cc, K, R, S, stride, pad, groups,
                             K if ldy is None else int(ldy), fmt(f_in), _ptr(frac_w), int(frac_w_range[0]),
                             int(frac_w_range[1]), fmt(f_out), int(bool(relu)), _stream(stream))
    _check(st, "dfq_conv_q_pc")
    return y, acc


def conv_q_add(x: torch.Tensor, w: torch.Tensor, b: Optional[torch.Tensor], other: torch.Tensor, f_in: int, f_w: int,
               f_mid: int, relu_mid: bool, f_other: int, f_out: int, relu_out: bool, stride: int = 1, pad: int = 0,
               groups: int = 1, out: Optional[torch.Tensor] = None, stream=None):
    """Convolution and the element-wise add behind it in one kernel: what conv_q(..., f_mid, relu_mid)
    followed by eltwise_q(that, f_mid, other, f_other, f_out, relu_out) gives.  Returns the int8
    result, or None when no fused kernel covers the call (nothing was launched)."""
    _dev(x, torch.int8, "x"); _dev(w, torch.int8, "w"); _dev(other, torch.int8, "other")
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = x.shape
    K, R, S, Cg = w.shape
    if Cg * groups != Cc:
        raise DfqError(ESHAPE, "conv_q_add (weight shape does not match C/groups)")
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    if tuple(other.shape) != (N, P, Q, K):
        raise DfqError(ESHAPE, "conv_q_add (second operand's shape)")
    y = out if out is not None else torch.empty((N, P, Q, K), dtype=torch.int8, device=x.device)
    st = lib().dfq_conv_q_add(_ptr(x), _ptr(w), _ptr(b), _ptr(other), _ptr(y), N, H, W, Cc, K, R, S, stride, pad, groups,
                              K, K, fmt(f_in), fmt(f_w), fmt(f_mid), int(bool(relu_mid)), fmt(f_other), fmt(f_out),
                              int(bool(relu_out)), _stream(stream))
    if st == EUNSUPPORTED:
        return None
    _check(st, "dfq_conv_q_add")
    return y


def conv_q_add_lazy(x: torch.Tensor, w: torch.Tensor, b: Optional[torch.Tensor], other: torch.Tensor, f_in: int, f_w: int,
                    f_other: int, f_out: int, relu_out: bool, stride: int = 1, pad: int = 0, groups: int = 1,
                    out: Optional[torch.Tensor] = None, stream=None):
    """Convolution + element-wise add with a single rounding (the accumulator and `other` summed at the accumulator's
    scale).  Returns the int8 result, or None when no fused kernel covers the call (nothing was launched)."""
    _dev(x, torch.int8, "x"); _dev(w, torch.int8, "w"); _dev(other, torch.int8, "other")
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = x.shape
    K, R, S, Cg = w.shape
    if Cg * groups != Cc:
        raise DfqError(ESHAPE, "conv_q_add_lazy (weight shape does not match C/groups)")
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    if tuple(other.shape) != (N, P, Q, K):
        raise DfqError(ESHAPE, "conv_q_add_lazy (second operand's shape)")
    y = out if out is not None else torch.empty((N, P, Q, K), dtype=torch.int8, device=x.device)
    st = lib().dfq_conv_q_add_lazy(_ptr(x), _ptr(w), _ptr(b), _ptr(other), _ptr(y), N, H, W, Cc, K, R, S, stride, pad, groups,
                                   K, K, fmt(f_in), fmt(f_w), fmt(f_other), fmt(f_out), int(bool(relu_out)), _stream(stream))
    if st == EUNSUPPORTED:
        return None
    _check(st, "dfq_conv_q_add_lazy")
    return y


def quantize_conv_q(x: torch.Tensor, w: torch.Tensor, b: Optional[torch.Tensor], f_in: int, f_w: int, f_out: int, stride: int,
                    pad: int, relu: bool, out: Optional[torch.Tensor] = None, stream=None):
    """Float images converted at f_in inside the first layer's kernel.  Returns the int8 result, or None when no fused
    kernel covers the call (nothing was launched)."""
    _dev(x, torch.float32, "x"); _dev(w, torch.int8, "w")
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = x.shape
    K, R, S, Cg = w.shape
    if Cg != Cc:
        raise DfqError(ESHAPE, "quantize_conv_q (weight shape does not match C)")
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    y = out if out is not None else torch.empty((N, P, Q, K), dtype=torch.int8, device=x.device)
    st = lib().dfq_quantize_conv_q(_ptr(x), _ptr(w), _ptr(b), _ptr(y), N, H, W, Cc, K, R, S, stride, pad, 1, K, fmt(f_in), fmt(f_w),
                                   fmt(f_out), int(bool(relu)), _stream(stream))
    if st == EUNSUPPORTED:
        return None
    _check(st, "dfq_quantize_conv_q")
    return y


def conv_q_maxpool(x: torch.Tensor, w: torch.Tensor, b: Optional[torch.Tensor], f_in: int, f_w, f_out: int, stride: int,
                   pad: int, relu: bool, pool_k: int = 3, pool_stride: int = 2, pool_pad: int = 1,
                   out: Optional[torch.Tensor] = None, stream=None, frac_w_range=None):
    """Convolution + max-pooling in one kernel; x int8 codes, or float32 images that are converted at f_in on the way in
    (dfq_quantize_conv_q_maxpool).  Returns the pooled int8 tensor, or None when no fused kernel covers the call (nothing
    was launched)."""
    from_float = x.dtype == torch.float32
    _dev(x, torch.float32 if from_float else torch.int8, "x"); _dev(w, torch.int8, "w")
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = x.shape
    K, R, S, Cg = w.shape
    if Cg != Cc:
        raise DfqError(ESHAPE, "conv_q_maxpool (weight shape does not match C)")
    P, Q = conv_out_hw(H, W, R, S, stride, pad)
    PP, PQ = conv_out_hw(P, Q, pool_k, pool_k, pool_stride, pool_pad)
    y = out if out is not None else torch.empty((N, PP, PQ, K), dtype=torch.int8, device=x.device)
    if isinstance(f_w, torch.Tensor):
        # one weight format per output channel: f_w a device int32 array of K entries, frac_w_range the bounds of its entries
        _dev(f_w, torch.int32, "frac_w")
        lo, hi = frac_w_range
        fn = lib().dfq_quantize_conv_q_pc_maxpool if from_float else lib().dfq_conv_q_pc_maxpool
        st = fn(_ptr(x), _ptr(w), _ptr(b), _ptr(y), N, H, W, Cc, K, R, S, stride, pad, 1, K, fmt(f_in), _ptr(f_w), int(lo), int(hi),
                fmt(f_out), int(bool(relu)), pool_k, pool_stride, pool_pad, _stream(stream))
    else:
        fn = lib().dfq_quantize_conv_q_maxpool if from_float else lib().dfq_conv_q_maxpool
        st = fn(_ptr(x), _ptr(w), _ptr(b), _ptr(y), N, H, W, Cc, K, R, S, stride, pad, 1, K, fmt(f_in), fmt(f_w),
                fmt(f_out), int(bool(relu)), pool_k, pool_stride, pool_pad, _stream(stream))
    if st == EUNSUPPORTED:
        return None
    _check(st, "dfq_conv_q_maxpool")
    return y


def conv_q_pc_add(x: torch.Tensor, w: torch.Tensor, b: Optional[torch.Tensor], other: torch.Tensor, f_in: int,
                  frac_w: torch.Tensor, frac_w_range, f_mid: int, relu_mid: bool, f_other: int, f_out: int, relu_out: bool,
                  out: Optional[torch.Tensor] = None, stream=None):
    """conv_q_add with one weight format per output channel (1x1, stride 1, no padding).  Returns the int8
    result, or None when no fused kernel covers the call (nothing was launched)."""
    _dev(x, torch.int8, "x"); _dev(w, torch.int8, "w"); _dev(other, torch.int8, "other"); _dev(frac_w, torch.int32, "frac_w")
    if b is not None:
        _dev(b, torch.int32, "b")
    N, H, W, Cc = x.shape
    K, R, S, Cg = w.shape
    if Cg != Cc or tuple(frac_w.shape) != (K,):
        raise DfqError(ESHAPE, "conv_q_pc_add (weight or format shape)")
    P, Q = conv_out_hw(H, W, R, S, 1, 0)
    if tuple(other.shape) != (N, P, Q, K):
        raise DfqError(ESHAPE, "conv_q_pc_add (second operand's shape)")
    y = out if out is not None else torch.empty((N, P, Q, K), dtype=torch.int8, device=x.device)
    st = lib().dfq_conv_q_pc_add(_ptr(x), _ptr(w), _ptr(b), _ptr(other), _ptr(y), N, H, W, Cc, K, R, S, 1, 0, 1, K, K,
                                 fmt(f_in), _ptr(frac_w), int(frac_w_range[0]), int(frac_w_range[1]), fmt(f_mid),
                                 int(bool(relu_mid)), fmt(f_other), fmt(f_out), int(bool(relu_out)), _stream(stream))
    if st == EUNSUPPORTED:
        return None
    _check(st, "dfq_conv_q_pc_add")
    return y


def conv_q_select(N, H, W, Cc, K, R, S, stride, pad, groups) -> int:
    return int(lib().dfq_conv_q_select(N, H, W, Cc, K, R, S, stride, pad, groups))


def eltwise_q(a: torch.Tensor, f_a: int, b: torch.Tensor, f_b: int, f_y: int, relu: bool = False,
              out: Optional[torch.Tensor] = None, want_y: bool = True, want_acc: bool = False, stream=None):
    _dev(a, torch.int8, "a"); _dev(b, torch.int8, "b")
    if a.shape != b.shape:
        raise DfqError(ESHAPE, "eltwise_q (shapes differ)")
    y = out if out is not None else (torch.empty_like(a) if want_y else None)
    acc = torch.empty(a.shape, dtype=torch.int32, device=a.device) if want_acc else None
    st = lib().dfq_eltwise_q(_ptr(a), fmt(f_a), _ptr(b), fmt(f_b), _ptr(y), fmt(f_y), _ptr(acc), a.numel(),
                             int(bool(relu)), _stream(stream))
    _check(st, "dfq_eltwise_q")
    return y, acc


def concat_q_into(xs: Sequence[torch.Tensor], fs: Sequence[int], f_y: int, out: torch.Tensor, ch_off: int, stream=None):
    """Branches xs (each [..., C_i]) rescaled into the channels ch_off .. ch_off + sum C_i of the wider tensor `out`."""
    for i, x in enumerate(xs):
        _dev(x, torch.int8, f"xs[{i}]")
    _dev(out, torch.int8, "out")
    lead = tuple(xs[0].shape[:-1])
    if any(tuple(x.shape[:-1]) != lead for x in xs) or tuple(out.shape[:-1]) != lead:
        raise DfqError(ESHAPE, "concat_q_into (pixel grids differ)")
    Cs = [int(x.shape[-1]) for x in xs]
    if ch_off < 0 or ch_off + sum(Cs) > out.shape[-1]:
        raise DfqError(ESHAPE, "concat_q_into (slice outside the destination)")
    nb = len(xs)
    ptrs = (C.c_void_p * nb)(*[x.data_ptr() for x in xs])
    st = lib().dfq_concat_q_into(nb, ptrs, (C.c_int * nb)(*Cs), (Fmt * nb)(*[fmt(f) for f in fs]), out.data_ptr() + int(ch_off),
                                 int(out.shape[-1]), fmt(f_y), out.numel() // out.shape[-1], _stream(stream))
    _check(st, "dfq_concat_q_into")
    return out


def concat_q(xs: Sequence[torch.Tensor], fs: Sequence[int], f_y: int, out: Optional[torch.Tensor] = None,
             stream=None) -> torch.Tensor:
    for i, x in enumerate(xs):
        _dev(x, torch.int8, f"xs[{i}]")
    lead = tuple(xs[0].shape[:-1])
    if any(tuple(x.shape[:-1]) != lead for x in xs):
        raise DfqError(ESHAPE, "concat_q (pixel grids differ)")
    Cs = [int(x.shape[-1]) for x in xs]
    pixels = 1
    for d in lead:
        pixels *= int(d)
    y = out if out is not None else torch.empty(lead + (sum(Cs),), dtype=torch.int8, device=xs[0].device)
    nb = len(xs)
    ptrs = (C.c_void_p * nb)(*[x.data_ptr() for x in xs])
    st = lib().dfq_concat_q(nb, ptrs, (C.c_int * nb)(*Cs), (Fmt * nb)(*[fmt(f) for f in fs]), _ptr(y), fmt(f_y),
                            pixels, _stream(stream))
    _check(st, "dfq_concat_q")
    return y


def pool_q(x: torch.Tensor, mode: str, k: int, stride: int, pad: int, f_in: int, f_out: int,
           out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    _dev(x, torch.int8, "x")
    N, H, W, Cc = x.shape
    P, Q = conv_out_hw(H, W, k, k, stride, pad)
    y = out if out is not None else torch.empty((N, max(P, 0), max(Q, 0), Cc), dtype=torch.int8, device=x.device)
    st = lib().dfq_pool_q(_ptr(x), _ptr(y), {"max": POOL_MAX, "avg": POOL_AVG}[mode], N, H, W, Cc, k, stride, pad,
                          fmt(f_in), fmt(f_out), _stream(stream))
    _check(st, "dfq_pool_q")
    return y


# ---- calibration building blocks ------------------------------------------------------ #
def absmax_f32(x: torch.Tensor, out_dev: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Returns a one-element float32 device tensor (no synchronization)."""
    _dev(x, torch.float32, "x")
    out = out_dev if out_dev is not None else torch.empty(1, dtype=torch.float32, device=x.device)
    _check(lib().dfq_absmax_f32(_ptr(x), x.numel(), _ptr(out), _stream(stream)), "dfq_absmax_f32")
    return out


def absmax_i32(x: torch.Tensor, relu: bool = False, out_dev: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Returns a one-element device tensor holding the maximum as uint32 bits (stored in int64-free
    int32 storage; read it with ``absmax_i32_value``)."""
    _dev(x, torch.int32, "x")
    out = out_dev if out_dev is not None else torch.empty(1, dtype=torch.int32, device=x.device)
    _check(lib().dfq_absmax_i32(_ptr(x), x.numel(), int(bool(relu)), _ptr(out), _stream(stream)), "dfq_absmax_i32")
    return out


def absmax_f32_rows(x: torch.Tensor, stream=None) -> torch.Tensor:
    """max |.| of every row of a float32 [rows, ...] tensor: float32 device tensor [rows] (no synchronization)."""
    _dev(x, torch.float32, "x")
    rows = int(x.shape[0])
    out = torch.zeros(rows, dtype=torch.float32, device=x.device)
    _check(lib().dfq_absmax_f32_rows(_ptr(x), rows, x.numel() // max(rows, 1), _ptr(out), _stream(stream)),
           "dfq_absmax_f32_rows")
    return out


def quantize_rows(x: torch.Tensor, frac: torch.Tensor, stream=None) -> torch.Tensor:
    """int8 codes of a float32 [rows, ...] tensor, row r at fractional length frac[r] (int32 device tensor)."""
    _dev(x, torch.float32, "x"); _dev(frac, torch.int32, "frac")
    rows = int(x.shape[0])
    q = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _check(lib().dfq_quantize_rows(_ptr(x), _ptr(q), rows, x.numel() // max(rows, 1), _ptr(frac), _stream(stream)),
           "dfq_quantize_rows")
    return q


def quantize_i32_rows(x: torch.Tensor, frac: torch.Tensor, frac_add: int, stream=None) -> torch.Tensor:
    """int32 codes of a float32 [rows, ...] tensor, row r at fractional length frac[r] + frac_add."""
    _dev(x, torch.float32, "x"); _dev(frac, torch.int32, "frac")
    rows = int(x.shape[0])
    q = torch.empty(x.shape, dtype=torch.int32, device=x.device)
    _check(lib().dfq_quantize_i32_rows(_ptr(x), _ptr(q), rows, x.numel() // max(rows, 1), _ptr(frac), int(frac_add),
                                       _stream(stream)), "dfq_quantize_i32_rows")
    return q


def fold_scale(w: torch.Tensor, b: Optional[torch.Tensor], scale: torch.Tensor, shift: Optional[torch.Tensor], stream=None):
    """Float weights [rows, ...] and bias [rows] with the per-row affine layer behind the convolution folded in:
    (w * scale[row], b * scale + shift) as new float32 device tensors."""
    _dev(w, torch.float32, "w"); _dev(scale, torch.float32, "scale")
    rows = int(w.shape[0])
    for t_, name in ((b, "b"), (shift, "shift")):
        if t_ is not None:
            _dev(t_, torch.float32, name)
            if tuple(t_.shape) != (rows,):
                raise DfqError(ESHAPE, "fold_scale (one bias / shift per row)")
    if tuple(scale.shape) != (rows,):
        raise DfqError(ESHAPE, "fold_scale (one scale per row)")
    w_out = torch.empty_like(w)
    b_out = torch.empty(rows, dtype=torch.float32, device=w.device)
    _check(lib().dfq_fold_scale_f32(_ptr(w), _ptr(b), rows, w.numel() // max(rows, 1), _ptr(scale), _ptr(shift), _ptr(w_out),
                                    _ptr(b_out), _stream(stream)), "dfq_fold_scale_f32")
    return w_out, b_out


def absmax_i32_channels(x: torch.Tensor, relu: bool = False, out_dev: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Per-channel maxima of |x| over the leading axes of an int32 [..., K] tensor: K uint32 words in
    an int32 device tensor (no synchronization; read with ``absmax_i32_channels_value``)."""
    _dev(x, torch.int32, "x")
    K = int(x.shape[-1])
    out = out_dev if out_dev is not None else torch.empty(K, dtype=torch.int32, device=x.device)
    _check(lib().dfq_absmax_i32_channels(_ptr(x), x.numel() // K, K, int(bool(relu)), _ptr(out), _stream(stream)),
           "dfq_absmax_i32_channels")
    return out


def absmax_i32_channels_value(out_dev: torch.Tensor):
    """Host values (numpy uint32 [K]) of an absmax_i32_channels result (synchronizes)."""
    return out_dev.cpu().numpy().view("uint32")


HIST_BINS = 2048


def hist_shift(max_abs: int) -> int:
    """The smallest shift with (max_abs >> shift) < HIST_BINS."""
    j = int(lib().dfq_hist_shift(int(max_abs)))
    if j < 0:
        raise DfqError(EINVAL, "dfq_hist_shift")
    return j


def hist_i32(x: torch.Tensor, shift: int, relu: bool = False, out_dev: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Counts of (|x| >> shift) per bin: HIST_BINS uint32 words in an int32 device tensor (no synchronization)."""
    _dev(x, torch.int32, "x")
    out = out_dev if out_dev is not None else torch.empty(HIST_BINS, dtype=torch.int32, device=x.device)
    _check(lib().dfq_hist_i32(_ptr(x), x.numel(), int(bool(relu)), int(shift), _ptr(out), _stream(stream)), "dfq_hist_i32")
    return out


def threshold_search(hist_host, shift: int, max_abs: int):
    """Algorithm 1 on a host histogram (numpy uint32, at least (max_abs >> shift) + 1 entries): (gamma, delta)."""
    import numpy as np
    nb = (int(max_abs) >> int(shift)) + 1
    h = np.ascontiguousarray(np.asarray(hist_host).view(np.uint32)[:nb])
    g, d = C.c_int64(0), C.c_double(0.0)
    _check(lib().dfq_threshold_search(h.ctypes.data_as(C.c_void_p), nb, int(shift), int(max_abs), C.byref(g), C.byref(d)),
           "dfq_threshold_search")
    return int(g.value), float(d.value)


def absmax_i32_value(out_dev: torch.Tensor) -> int:
    """Host value of an absmax_i32 result (synchronizes)."""
    return int(out_dev.cpu().numpy().view("uint32")[0])


def fmt_from_absmax_f32(gamma: float) -> int:
    f = Fmt()
    _check(lib().dfq_fmt_from_absmax_f32(float(gamma), C.byref(f)), "dfq_fmt_from_absmax_f32")
    return int(f.frac)


def np_frac_from_absmax_f32(gamma: float, nbits: int, p: int) -> int:
    f = C.c_int32()
    _check(lib().dfq_np_frac_from_absmax_f32(float(gamma), int(nbits), int(p), C.byref(f)), "dfq_np_frac_from_absmax_f32")
    return int(f.value)


def fmt_from_absmax_i32(m: int, acc_frac: int) -> int:
    f = Fmt()
    _check(lib().dfq_fmt_from_absmax_i32(int(m), int(acc_frac), C.byref(f)), "dfq_fmt_from_absmax_i32")
    return int(f.frac)


def fmt_from_absmax_i32_channels(m_host, f_in: int, frac_w_host) -> int:
    """Output format of a layer with one weight format per output channel from the per-channel thresholds
    (numpy uint32 [K], as ``absmax_i32_channels_value`` returns them) and the per-channel weight formats
    (numpy int32 [K])."""
    import numpy as np
    m = np.ascontiguousarray(m_host, np.uint32)
    fw = np.ascontiguousarray(frac_w_host, np.int32)
    if m.shape != fw.shape or m.ndim != 1:
        raise DfqError(ESHAPE, "fmt_from_absmax_i32_channels (one threshold and one format per channel)")
    f = Fmt()
    _check(lib().dfq_fmt_from_absmax_i32_channels(m.ctypes.data_as(C.c_void_p), int(m.shape[0]), int(f_in),
                                                  fw.ctypes.data_as(C.c_void_p), C.byref(f)), "dfq_fmt_from_absmax_i32_channels")
    return int(f.frac)


# ---- closed forms ------------------------------------------------------------------- #
def beta_max(n, p): return int(lib().dfq_beta_max(n, p))
def mac_acc_bits(N, bx, ex, by, ey): return int(lib().dfq_mac_acc_bits(N, bx, ex, by, ey))
def mac_max_len(q, bx, ex, by, ey): return int(lib().dfq_mac_max_len(q, bx, ex, by, ey))
def add_acc_bits(N, bx, ex): return int(lib().dfq_add_acc_bits(N, bx, ex))
def add_max_len(q, bx, ex): return int(lib().dfq_add_max_len(q, bx, ex))
