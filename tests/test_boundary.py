"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, validates arguments before launching anything, and its pure host functions
agree with the hand-worked closed forms."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dfq.h")
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


@pytest.fixture(scope="module")
def B():
    from paper_1805_07941_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_1805_07941_amd import build
        build.build(force=True)
    binding.lib()
    return binding


def _declared(header):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dfq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(B):
    declared = _declared(HEADER)
    assert len(declared) >= 19
    L = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), f"{name} declared in dfq.h but not exported"
    assert sorted(B.EXPORTS) == declared
    # every header under include/ is covered: the only other one declares the benchmark aid of libdfq_probe.so
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["dfq.h", "dfq_probe.h"]
    from paper_1805_07941_amd import probe
    declared_p = _declared(os.path.join(ROOT, "include", "dfq_probe.h"))
    LP = C.CDLL(probe.LIB_PATH)
    for name in declared_p:
        assert hasattr(LP, name), f"{name} declared in dfq_probe.h but not exported"
        assert not hasattr(L, name), f"{name} is a measurement aid and must stay out of libdfq.so"
    assert sorted(probe.EXPORTS) == declared_p
    P = probe.lib()
    assert P.dfq_probe_mfma_rate(None, 1 << 20, 2 << 20, 1, 1, None, None) == 1
    assert P.dfq_probe_mfma_rate(1 << 20, 2 << 20, 3 << 20, 0, 1, None, None) == 1              # no workgroups
    assert P.dfq_probe_mfma_rate(1 << 20, (2 << 20) + 4, 3 << 20, 1, 1, None, None) == 1        # alignment


def test_status_strings(B):
    assert B.status_string(B.OK) == "ok"
    assert len({B.status_string(s) for s in range(6)}) == 6


def test_closed_forms_match_golden(B):
    fns = {"beta_max": B.beta_max, "mac_bits": B.mac_acc_bits, "mac_len": B.mac_max_len,
           "add_bits": B.add_acc_bits, "add_len": B.add_max_len}
    n = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        kind, *vals = line.split()
        *args, want = [int(v) for v in vals]
        assert fns[kind](*args) == want, line
        n += 1
    assert n >= 20
    assert B.beta_max(8, 9) == -1 and B.mac_acc_bits(0, 1, 0, 1, 0) == -1


def test_format_from_thresholds(B):
    f = B.fmt_from_absmax_f32
    assert f(1.0) == 6 and f(1.99) == 5 and f(0.0) == 32 and f(127.0) == 0 and f(127.5) == -1 and f(1e30) == -32
    for bad in (float("nan"), float("inf"), -1.0):
        with pytest.raises(B.DfqError):
            f(bad)
    g = B.fmt_from_absmax_i32
    assert g(0, 11) == 11 and g(127, 11) == 11 and g(128, 11) == 10 and g(254, 11) == 10 and g(255, 11) == 9
    assert g(127 * 128, 11) == 4 and g(127 * 128 + 1, 11) == 3 and g(1, 40) == 32 and g(2 ** 31, -20) == -32
    with pytest.raises(B.DfqError):
        g(-1, 0)
    # one weight format per output channel: the smallest of the per-channel results
    import oracle as orc
    rng = np.random.default_rng(17)
    for K in (1, 7, 64):
        m = rng.integers(0, 2 ** 31, K).astype(np.uint32)
        m[0] = 0
        fw = rng.integers(-3, 12, K).astype(np.int32)
        for f_in in (-2, 4, 9):
            want = min(orc.frac_from_absmax_i32(int(m[k]), f_in + int(fw[k])) for k in range(K))
            assert B.fmt_from_absmax_i32_channels(m, f_in, fw) == want
    assert B.fmt_from_absmax_i32_channels(np.array([127, 128], np.uint32), 4, np.array([7, 7], np.int32)) == 10
    assert B.fmt_from_absmax_i32_channels(np.array([127, 128], np.uint32), 4, np.array([7, 9], np.int32)) == 11
    with pytest.raises(B.DfqError):
        B.fmt_from_absmax_i32_channels(np.array([1], np.uint32), 0, np.array([40], np.int32))
    # bin width of the histogram of Algorithm 1
    assert [B.hist_shift(v) for v in (0, 2047, 2048, 4095, 4096, 2 ** 31)] == [0, 0, 1, 1, 2, 21]
    assert B.lib().dfq_hist_shift(-1) == -1


def _conv(B, **kw):
    a = dict(x=1 << 20, w=2 << 20, b=None, y=3 << 20, acc=None, N=1, H=8, W=8, Cc=16, K=16, R=3, S=3, stride=1, pad=1,
             groups=1, ldy=16, fi=4, fw=7, fo=4, bits=8)
    a.update(kw)
    fm = lambda f: B.Fmt(a["bits"], f)
    return B.lib().dfq_conv_q(a["x"], a["w"], a["b"], a["y"], a["acc"], a["N"], a["H"], a["W"], a["Cc"], a["K"], a["R"],
                              a["S"], a["stride"], a["pad"], a["groups"], a["ldy"], fm(a["fi"]), fm(a["fw"]), fm(a["fo"]),
                              0, None)


def test_conv_q_rejects_bad_arguments_before_launching(B):
    # (pointers are fake non-null addresses: every case below must fail in validation)
    assert _conv(B, x=None) == B.EINVAL
    assert _conv(B, y=None) == B.EINVAL                       # neither y nor acc_out
    assert _conv(B, N=-1) == B.EINVAL
    assert _conv(B, Cc=0) == B.ESHAPE
    assert _conv(B, groups=3) == B.ESHAPE                     # C % groups
    assert _conv(B, K=20, groups=8, Cc=16, ldy=20) == B.ESHAPE  # K % groups
    assert _conv(B, H=2, W=2, R=5, S=5, pad=0) == B.ESHAPE    # empty output
    assert _conv(B, ldy=8) == B.ESHAPE                        # ldy < K
    assert _conv(B, stride=0) == B.ESHAPE
    assert _conv(B, bits=4) == B.EFMT
    assert _conv(B, fi=33) == B.EFMT
    assert _conv(B, Cc=16384, R=3, S=3) == B.EUNSUPPORTED     # 9*16384 products exceed Eq. 9's bound for 32 bits
    assert _conv(B, y=1 << 20) == B.EINVAL                    # output aliases the input
    assert _conv(B, N=0) == B.OK                              # empty batch: nothing to do


def test_conv_q_maxpool_rejects_bad_arguments_before_launching(B):
    L = B.lib()
    f = B.fmt

    def call(x=1 << 20, w=2 << 20, y=3 << 20, N=1, H=64, W=64, C=3, K=64, R=7, S=7, stride=2, pad=3, groups=1, ldy=64, fi=4, fw=7,
             fo=4, k=3, ps=2, pp=1):
        return L.dfq_conv_q_maxpool(x, w, None, y, N, H, W, C, K, R, S, stride, pad, groups, ldy, f(fi), f(fw), f(fo), 1, k, ps, pp, None)

    assert call(x=None) == B.EINVAL
    assert call(y=None) == B.EINVAL
    assert call(N=-1) == B.EINVAL
    assert call(C=0) == B.ESHAPE
    assert call(k=0) == B.ESHAPE
    assert call(pp=3) == B.ESHAPE                             # pooling pad >= window
    assert call(ldy=32) == B.ESHAPE                           # ldy < K
    assert call(fo=40) == B.EFMT
    assert call(y=1 << 20) == B.EINVAL                        # output aliases the input
    assert call(N=0) == B.OK                                  # empty batch: nothing to do
    # valid requests no fused kernel covers: nothing is launched
    assert call(k=2, ps=2, pp=0) == B.EUNSUPPORTED            # another pooling
    assert call(C=4) == B.EUNSUPPORTED                        # not a 3-channel first layer
    assert call(H=66) == B.EUNSUPPORTED                       # 33 output rows: the last window would hang over the image
    assert call(W=252) == B.EUNSUPPORTED                      # 63 pooled columns
    assert call(fo=12) == B.EUNSUPPORTED                      # rescale shift below 0
    assert call(ldy=72) == B.EUNSUPPORTED                     # output pixels not 16-byte aligned

    # the same call on float images
    def callf(x=1 << 20, y=3 << 20, N=1, H=64, W=64, fi=4):
        return L.dfq_quantize_conv_q_maxpool(x, 2 << 20, None, y, N, H, W, 3, 64, 7, 7, 2, 3, 1, 64, f(fi), f(7), f(4), 1, 3, 2, 1, None)

    assert callf(x=None) == B.EINVAL
    assert callf(fi=-40) == B.EFMT
    assert callf(y=(1 << 20) + 4 * 64 * 64 * 3 - 16) == B.EINVAL   # the output begins inside the float images (4 bytes per element)
    assert callf(N=0) == B.OK
    assert callf(x=(1 << 20) + 4) == B.EUNSUPPORTED           # images not 16-byte aligned
    assert callf(H=66) == B.EUNSUPPORTED

    # float images into a first layer without pooling
    def callq(x=1 << 20, y=3 << 20, N=1, K=32, W=64, ldy=None, fo=4):
        return L.dfq_quantize_conv_q(x, 2 << 20, None, y, N, 64, W, 3, K, 3, 3, 2, 1, 1, K if ldy is None else ldy, f(4), f(7), f(fo), 1, None)

    assert callq(x=None) == B.EINVAL
    assert callq(y=None) == B.EINVAL
    assert callq(ldy=16) == B.ESHAPE
    assert callq(fo=40) == B.EFMT
    assert callq(y=(1 << 20) + 64) == B.EINVAL                # output inside the images
    assert callq(N=0) == B.OK
    assert callq(K=64) == B.EUNSUPPORTED                      # float images: 32 output channels only
    assert callq(W=72) == B.EUNSUPPORTED                      # 36 output columns
    assert callq(x=(1 << 20) + 8) == B.EUNSUPPORTED

    # one weight format per output channel
    def callpc(fw=4 << 20, lo=3, hi=9, fo=4, fn=L.dfq_conv_q_pc_maxpool):
        return fn(1 << 20, 2 << 20, None, 3 << 20, 1, 64, 64, 3, 64, 7, 7, 2, 3, 1, 64, f(4), fw, lo, hi, f(fo), 1, 3, 2, 1, None)

    for fn in (L.dfq_conv_q_pc_maxpool, L.dfq_quantize_conv_q_pc_maxpool):
        assert callpc(fw=None, fn=fn) == B.EINVAL
        assert callpc(fw=(4 << 20) + 2, fn=fn) == B.EINVAL        # format array not 4-byte aligned
        assert callpc(lo=9, hi=3, fn=fn) == B.EFMT
        assert callpc(hi=40, fn=fn) == B.EFMT
        assert callpc(lo=3, hi=24, fn=fn) == B.EUNSUPPORTED       # shifts 4 + 24 - 4 > 23
        assert callpc(lo=-1, hi=5, fn=fn) == B.EUNSUPPORTED       # a shift below 0


def test_conv_np_rejects_bad_arguments_before_launching(B):
    """(fake non-null addresses, 16-byte aligned and far apart: every case below must fail in validation)"""
    L = B.lib()

    def call(variant=B.CONV_AUTO, xh=1 << 20, xl=2 << 20, wh=3 << 20, wl=4 << 20, b=None, y=6 << 20, yh=7 << 20, yl=8 << 20,
             N=1, H=8, W=8, Cc=64, K=16, R=3, S=3, stride=1, pad=1, groups=1, fx=8, fw=8, fy=3, p_y=4, relu=0):
        return L.dfq_conv_np_variant(variant, xh, xl, wh, wl, b, y, yh, yl, N, H, W, Cc, K, R, S, stride, pad, groups, fx, fw, fy, p_y,
                                     relu, None)

    assert call(xh=None) == B.EINVAL and call(wl=None) == B.EINVAL
    assert call(y=None, yh=None, yl=None) == B.EINVAL              # no output at all
    assert call(yl=None) == B.EINVAL                               # one plane without the other
    assert call(N=-1) == B.EINVAL
    assert call(Cc=0) == B.ESHAPE and call(groups=3) == B.ESHAPE and call(H=1, W=1, pad=0) == B.ESHAPE and call(stride=0) == B.ESHAPE
    assert call(p_y=3) == B.EFMT and call(p_y=8) == B.EFMT         # (8, 3) integers need 18 bits: not this path
    assert call(fx=33) == B.EFMT
    assert call(fx=32, fw=32, fy=-32) == B.EFMT                    # shift 96
    assert call(fx=-32, fw=0, fy=0) == B.EFMT                      # shift -32
    assert call(y=1 << 20) == B.EINVAL and call(yh=6 << 20) == B.EINVAL      # output over input, output over output
    assert call(variant=B.CONV_MFMA, Cc=48) == B.EUNSUPPORTED      # reduction not in whole 64-byte steps
    assert call(variant=B.CONV_MFMA, K=24) == B.EUNSUPPORTED
    assert call(variant=B.CONV_MFMA, groups=2) == B.EUNSUPPORTED
    assert call(variant=B.CONV_MFMA, xl=(2 << 20) + 4) == B.EUNSUPPORTED     # alignment
    assert call(variant=B.CONV_MFMA, Cc=1472, R=3, S=3) == B.EUNSUPPORTED    # 13248 terms: the int32 partial sums could overflow
    assert call(variant=B.CONV_DEPTHWISE) == B.EINVAL
    assert call(N=0) == B.OK
    assert L.dfq_np_digits(1 << 20, 16, 3, 2 << 20, 3 << 20, None) == B.EFMT
    assert L.dfq_np_digits(None, 16, 4, 2 << 20, 3 << 20, None) == B.EINVAL
    assert L.dfq_np_digits(1 << 20, 16, 4, 1 << 20, 3 << 20, None) == B.EINVAL     # in place
    assert L.dfq_np_digits(1 << 20, 0, 4, 2 << 20, 3 << 20, None) == B.OK


def test_eltwise_np_rejects_bad_arguments_before_launching(B):
    L = B.lib()

    def call(ah=1 << 20, al=2 << 20, fa=5, bh=3 << 20, bl=4 << 20, fb=5, y=5 << 20, yh=6 << 20, yl=7 << 20, fy=4, p_y=4, n=1000, relu=0):
        return L.dfq_eltwise_np(ah, al, fa, bh, bl, fb, y, yh, yl, fy, p_y, n, relu, None)

    assert call(ah=None) == B.EINVAL and call(bl=None) == B.EINVAL
    assert call(y=None, yh=None, yl=None) == B.EINVAL and call(yh=None) == B.EINVAL
    assert call(y=1 << 20) == B.EINVAL and call(yh=5 << 20) == B.EINVAL          # output over input, output over output
    assert call(p_y=3) == B.EFMT and call(p_y=8) == B.EFMT
    assert call(fa=33) == B.EFMT
    assert call(fa=20, fb=1) == B.EFMT                                           # a 19-bit alignment: Eq. 12 would need more than 32 bits
    assert call(fa=0, fb=0, fy=17) == B.EFMT and call(fa=32, fb=32, fy=0) == B.EFMT
    assert call(n=0) == B.OK and call(n=0, ah=None) == B.OK


def test_np_network_calls_reject_bad_arguments_before_launching(B):
    import ctypes as C
    L = B.lib()
    a = [1 << 20, 2 << 20, 3 << 20, 4 << 20]
    assert L.dfq_conv_np_absmax(*a, None, None, 1, 8, 8, 64, 16, 3, 3, 1, 1, 1, 0, None) == B.EINVAL          # no result word
    assert L.dfq_conv_np_absmax(*a, None, (9 << 20) + 4, 1, 8, 8, 64, 16, 3, 3, 1, 1, 1, 0, None) == B.EINVAL  # misaligned
    assert L.dfq_conv_np_absmax(None, *a[1:], None, 9 << 20, 1, 8, 8, 64, 16, 3, 3, 1, 1, 1, 0, None) == B.EINVAL
    assert L.dfq_conv_np_absmax(*a, None, 9 << 20, 1, 8, 8, 64, 16, 3, 3, 0, 1, 1, 0, None) == B.ESHAPE
    assert L.dfq_eltwise_np_absmax(a[0], a[1], 5, a[2], a[3], 5, None, 100, 0, None) == B.EINVAL
    assert L.dfq_eltwise_np_absmax(a[0], a[1], 20, a[2], a[3], 1, 9 << 20, 100, 0, None) == B.EFMT
    assert L.dfq_eltwise_np_absmax(None, a[1], 5, a[2], a[3], 5, 9 << 20, 100, 0, None) == B.EINVAL
    out = C.c_int32()
    assert L.dfq_np_frac_from_absmax_u64(5, 0, 8, 4, None) == B.EINVAL
    assert L.dfq_np_frac_from_absmax_u64(5, 0, 8, 9, C.byref(out)) == B.EFMT
    assert L.dfq_np_frac_from_absmax_u64(5, 200, 8, 4, C.byref(out)) == B.EFMT
    import oracle.npnet as NN
    import oracle.npfmt as F
    for p in (4, 5, 7):
        bm = F.beta_max(8, p)
        for m in [0, 1, bm - 1, bm, bm + 1, 2 * bm, 2 * bm + 1, 12345678, (1 << 36) + 5, bm << 20, (bm << 20) + 1, (1 << 63) + 1, (1 << 64) - 1]:
            for f_acc in [-40, -3, 0, 7, 20, 40, 100]:
                assert B.np_frac_from_absmax_u64(m, f_acc, 8, p) == NN.frac_from_absmax_int(m, f_acc, 8, p), (m, f_acc, p)

    def pool(xh=a[0], xl=a[1], y=5 << 20, yh=6 << 20, yl=7 << 20, mode=B.POOL_MAX, N=1, H=8, W=8, Cc=16, k=3, stride=2, pad=1, p=4):
        return L.dfq_pool_np(xh, xl, y, yh, yl, mode, N, H, W, Cc, k, stride, pad, p, None)

    assert pool(xh=None) == B.EINVAL and pool(y=None, yh=None, yl=None) == B.EINVAL and pool(yl=None) == B.EINVAL
    assert pool(y=a[0]) == B.EINVAL and pool(mode=7) == B.EINVAL
    assert pool(k=0) == B.ESHAPE and pool(k=17) == B.ESHAPE and pool(pad=3) == B.ESHAPE and pool(H=1, W=1, pad=0) == B.ESHAPE
    assert pool(mode=B.POOL_AVG) == B.EUNSUPPORTED and pool(p=3) == B.EFMT and pool(N=0) == B.OK
    assert L.dfq_stem_pack_x(None, 2 << 20, 1, 32, 32, 3, 7, 7, 3, None) == B.EINVAL
    assert L.dfq_stem_pack_x(1 << 20, 2 << 20, 1, 32, 32, 5, 7, 7, 3, None) == B.ESHAPE                        # five channels do not fit 16 bytes
    assert L.dfq_stem_pack_x(1 << 20, 2 << 20, 1, 32, 32, 3, 9, 9, 3, None) == B.ESHAPE
    assert L.dfq_stem_pack_x(1 << 20, (1 << 20) + 64, 1, 32, 32, 3, 7, 7, 3, None) == B.EINVAL                 # overlap
    assert L.dfq_stem_pack_x(1 << 20, 2 << 20, 0, 32, 32, 3, 7, 7, 3, None) == B.OK
    assert L.dfq_stem_pack_w(1 << 20, None, 64, 7, 7, 3, None) == B.EINVAL
    assert L.dfq_stem_pack_w(1 << 20, 2 << 20, 64, 7, 7, 5, None) == B.ESHAPE


def test_conv_np_add_rejects_bad_arguments_before_launching(B):
    L = B.lib()

    def call(xh=1 << 20, xl=2 << 20, wh=3 << 20, wl=4 << 20, b=None, oh=5 << 20, ol=6 << 20, yh=7 << 20, yl=8 << 20, N=1, H=8, W=8, Cc=64, K=64,
             R=1, S=1, stride=1, pad=0, groups=1, fx=10, fw=12, fm=10, relu_mid=0, fo=10, fy=9, p=4, relu_out=1):
        return L.dfq_conv_np_add(xh, xl, wh, wl, b, oh, ol, yh, yl, N, H, W, Cc, K, R, S, stride, pad, groups, fx, fw, fm, relu_mid, fo, fy, p,
                                 relu_out, None)

    assert call(yh=None) == B.EINVAL and call(oh=None) == B.EINVAL and call(xl=None) == B.EINVAL
    assert call(yh=5 << 20) == B.EINVAL and call(yl=1 << 20) == B.EINVAL                 # output over the other operand / the input
    assert call(stride=0) == B.ESHAPE and call(p=3) == B.EFMT and call(fo=33) == B.EFMT
    assert call(fo=29) == B.EFMT                                                         # a 19-bit alignment
    assert call(fw=2) == B.EUNSUPPORTED and call(fy=11) == B.EUNSUPPORTED and call(Cc=48) == B.EUNSUPPORTED
    assert call(oh=(5 << 20) + 4) == B.EUNSUPPORTED
    assert call(N=0) == B.OK


def test_np_frac_from_absmax_matches_the_oracle(B):
    import oracle.npfmt as F
    rng = np.random.default_rng(9)
    for g in list(np.exp(rng.uniform(-20, 20, 400)).astype(np.float32)) + [0.0, 1984.0, 1985.0, 127.0, 1e38]:
        for n, p in [(8, 4), (8, 3), (8, 7), (5, 1)]:
            assert B.np_frac_from_absmax_f32(float(g), n, p) == F.frac_from_absmax(float(g), n, p)
    out = C.c_int32()
    L = B.lib()
    assert L.dfq_np_frac_from_absmax_f32(-1.0, 8, 4, C.byref(out)) == B.EINVAL
    assert L.dfq_np_frac_from_absmax_f32(float("nan"), 8, 4, C.byref(out)) == B.EINVAL
    assert L.dfq_np_frac_from_absmax_f32(1.0, 9, 4, C.byref(out)) == B.EFMT
    assert L.dfq_np_frac_from_absmax_f32(1.0, 8, 4, None) == B.EINVAL


def test_other_calls_reject_bad_arguments(B):
    L = B.lib()
    f = B.fmt
    assert L.dfq_quantize(None, None, 0, f(4), None) == B.OK
    assert L.dfq_quantize(None, 1 << 20, 16, f(4), None) == B.EINVAL
    assert L.dfq_quantize(1 << 20, 2 << 20, 16, B.Fmt(16, 4), None) == B.EFMT
    assert L.dfq_quantize(1 << 20, (1 << 20) + 8, 16, f(4), None) == B.EINVAL        # overlap
    assert L.dfq_quantize_i32(1 << 20, 2 << 20, 16, 65, None) == B.EFMT
    assert L.dfq_quantize_np(1 << 20, 2 << 20, 16, 9, 4, 0, None) == B.EFMT                      # more than 8 bits
    assert L.dfq_quantize_np(1 << 20, 2 << 20, 16, 8, 8, 0, None) == B.EFMT                      # p > n - 1
    assert L.dfq_quantize_np(1 << 20, 2 << 20, 16, 8, 1, 0, None) == B.EFMT                      # six exponent bits
    assert L.dfq_quantize_np(1 << 20, 2 << 20, 16, 8, 4, 33, None) == B.EFMT
    assert L.dfq_quantize_np(1 << 20, None, 16, 8, 4, 0, None) == B.EINVAL
    assert L.dfq_quantize_np(None, None, 0, 8, 4, 0, None) == B.OK
    assert L.dfq_dequantize_np(1 << 20, (1 << 20) + 4, 16, 8, 4, 0, None) == B.EINVAL            # overlap
    assert L.dfq_dequantize_np(1 << 20, 2 << 20, 16, 1, 0, 0, None) == B.EFMT
    assert L.dfq_dequantize(1 << 20, 2 << 20, 16, f(-33), None) == B.EFMT
    assert L.dfq_eltwise_q(1 << 20, f(30), 2 << 20, f(0), 3 << 20, f(0), None, 16, 0, None) == B.EFMT
    assert L.dfq_eltwise_q(1 << 20, f(3), 2 << 20, f(3), None, f(3), None, 16, 0, None) == B.EINVAL
    assert L.dfq_eltwise_q(1 << 20, f(3), 2 << 20, f(3), 1 << 20, f(3), None, 16, 0, None) == B.EINVAL  # in place
    assert L.dfq_eltwise_q(None, f(3), None, f(3), None, f(3), None, 0, 0, None) == B.OK
    assert L.dfq_pool_q(1 << 20, 2 << 20, 2, 1, 8, 8, 4, 3, 2, 1, f(4), f(4), None) == B.EINVAL          # bad mode
    assert L.dfq_pool_q(1 << 20, 2 << 20, 0, 1, 8, 8, 4, 3, 2, 3, f(4), f(4), None) == B.ESHAPE          # pad >= k
    assert L.dfq_pool_q(1 << 20, 2 << 20, 0, 1, 8, 8, 4, 65, 1, 0, f(4), f(4), None) == B.ESHAPE         # k > 64
    assert L.dfq_pool_q(1 << 20, 2 << 20, 1, 1, 2, 2, 4, 3, 1, 0, f(4), f(4), None) == B.ESHAPE          # empty output
    assert L.dfq_concat_q(0, None, None, None, None, f(4), 4, None) == B.EINVAL
    ptrs = (C.c_void_p * 2)(1 << 20, 2 << 20)
    Cs = (C.c_int * 2)(4, 0)
    fs = (B.Fmt * 2)(f(3), f(4))
    assert L.dfq_concat_q(2, ptrs, Cs, fs, 3 << 20, f(3), 4, None) == B.ESHAPE
    Cs2 = (C.c_int * 2)(4, 8)
    assert L.dfq_concat_q_into(2, ptrs, Cs2, fs, 3 << 20, 11, f(3), 4, None) == B.ESHAPE              # row pitch below the channels
    assert L.dfq_concat_q_into(2, ptrs, Cs2, fs, None, 16, f(3), 4, None) == B.EINVAL
    assert L.dfq_concat_q_into(2, ptrs, Cs2, fs, (1 << 20) + 8, 16, f(3), 4, None) == B.EINVAL          # overlaps a branch
    assert L.dfq_concat_q_into(2, ptrs, Cs2, fs, None, 16, f(3), 0, None) == B.OK
    assert L.dfq_absmax_f32(1 << 20, 4, None, None) == B.EINVAL
    assert L.dfq_fold_scale_f32(1 << 20, None, 4, 8, None, None, 2 << 20, None, None) == B.EINVAL       # no scale
    assert L.dfq_fold_scale_f32(1 << 20, 5 << 20, 4, 8, 3 << 20, None, 2 << 20, None, None) == B.EINVAL  # bias but no b_out
    assert L.dfq_fold_scale_f32(1 << 20, None, 4, 8, 3 << 20, None, (1 << 20) + 16, None, None) == B.EINVAL   # partial overlap
    assert L.dfq_fold_scale_f32(None, None, 0, 8, None, None, None, None, None) == B.OK
    assert L.dfq_absmax_i32(None, 4, 0, 1 << 20, None) == B.EINVAL
    assert L.dfq_hist_i32(1 << 20, 4, 0, 32, 2 << 20, None) == B.EINVAL                               # shift
    assert L.dfq_hist_i32(1 << 20, 4, 0, 3, None, None) == B.EINVAL


def test_kernel_selection(B):
    s = B.conv_q_select
    assert s(1, 56, 56, 64, 64, 3, 3, 1, 1, 1) == B.CONV_MFMA
    assert s(1, 7, 7, 512, 2048, 1, 1, 1, 0, 1) == B.CONV_MFMA
    assert s(1, 8, 8, 0, 4, 1, 1, 1, 0, 1) == B.CONV_AUTO          # invalid geometry
    assert s(1, 8, 8, 20, 10, 2, 3, 1, 1, 5) == B.CONV_GROUPED     # groups of four channels
    assert s(1, 8, 8, 15, 10, 2, 3, 1, 1, 5) == B.CONV_DIRECT      # groups of three channels: no kernel but the direct one
    assert s(1, 8, 8, 64, 64, 3, 3, 1, 1, 64) == B.CONV_DEPTHWISE


def test_binding_fails_loudly_without_the_library(B, monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libdfq.so")
    with pytest.raises(RuntimeError):
        B.lib()


def test_threshold_search_is_host_code_and_matches_the_oracle(B):
    """dfq_threshold_search needs no GPU: Algorithm 1 on host histograms against the oracle's search,
    thresholds identical, measures to rounding."""
    import oracle as orc
    rng = np.random.default_rng(51)
    cases = []
    x = np.abs(rng.standard_normal(100000) * 3000).astype(np.int32); x[0] = 2_000_000
    cases.append(x)
    cases.append(rng.integers(0, 100000, 50000).astype(np.int32))
    cases.append(np.abs(rng.standard_normal(20000) * 40).astype(np.int32))          # fewer than 129 bins... or a few more
    cases.append((rng.exponential(500.0, 80000)).astype(np.int32))
    cases.append(rng.integers(-2 ** 31, 2 ** 31, 30000).astype(np.int32))
    cases.append(np.zeros(100, np.int32))
    for x in cases:
        counts, j, m = orc.hist_i32(x)
        want_g, want_d = orc.threshold_search(counts, j, m)
        got_g, got_d = B.threshold_search(counts.astype(np.uint32), j, m)
        assert got_g == want_g
        assert abs(got_d - want_d) <= 1e-12 * max(1.0, want_d)
    # the hand-worked histograms (derivation beside the oracle's pin of the same name)
    A = 10 ** 6
    counts = np.zeros(2048, np.uint32); counts[0] = A; counts[1] = A; counts[-1] = 1
    c0, c1 = A / (2 * A + 1.0), 2 * A / (2 * A + 1.0)
    g_, d_ = B.threshold_search(counts, 0, 2047)
    want = (c1 - c0) / 128 + (1 - c1) * (1919 + 1 / 128)
    assert g_ == 128 and abs(d_ - want) <= 1e-9 * want
    counts = np.zeros(256, np.uint32); counts[0] = 1000; counts[-1] = 1
    g_, d_ = B.threshold_search(counts, 0, 255)
    assert g_ == 255 and abs(d_ - (1 / 1001.0) * 129 / 255) <= 1e-9 * d_
    L = B.lib()
    h = (C.c_uint32 * 4)(1, 2, 3, 4)
    g = C.c_int64(0)
    assert L.dfq_threshold_search(h, 4, 0, 7, C.byref(g), None) == B.ESHAPE       # 7 >> 0 is not bin 3
    assert L.dfq_threshold_search(h, 4, 1, 7, C.byref(g), None) == B.OK and g.value == 7
    assert L.dfq_threshold_search(None, 4, 1, 7, C.byref(g), None) == B.EINVAL
