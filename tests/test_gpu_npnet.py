"""GPU parity of the pieces a whole network on (8, p) codes needs beyond convolution and add - calibration maxima, the
scale rule, pooling, the first layer's space-to-depth packing - and of calibration and inference of the ResNet-50-shaped
network on (8, 4) codes against the network oracle, tensor for tensor, through the C-ABI."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle.npconv as NC
import oracle.npfmt as F
import oracle.npnet as NN
import workloads as wl

from test_gpu_npconv import B, dev, host, digits_of, gaussian_codes, DEV          # noqa: F401  (B is a fixture)

pytestmark = pytest.mark.gpu


def planes(B, codes, p):
    return B.np_digits(dev(codes), p)


def beta_of(hl):
    return 64 * host(hl[0]).astype(np.int64) + host(hl[1])


@pytest.mark.parametrize("case", [
    # N, H, W, C, K, R, stride, pad, groups, relu, p
    (2, 9, 8, 64, 16, 3, 1, 1, 1, True, 4),
    (2, 9, 8, 64, 16, 3, 1, 1, 1, False, 4),
    (1, 7, 7, 8, 6, 3, 2, 1, 2, False, 5),
    (3, 5, 5, 128, 32, 1, 1, 0, 1, True, 4),
    (1, 4, 4, 512, 16, 3, 1, 1, 1, False, 4),          # sums beyond 32 bits
])
def test_conv_np_absmax(B, case):
    N, H, W, C, K, R, stride, pad, groups, relu, p = case
    rng = np.random.default_rng(sum(case))
    x = rng.integers(0, 256, (N, H, W, C)).astype(np.uint8) if C < 512 else np.full((N, H, W, C), 0x7f, np.uint8)
    w = rng.integers(0, 256, (K, R, R, C // groups)).astype(np.uint8) if C < 512 else np.full((K, R, R, C), 0xff if not relu else 0x7f, np.uint8)
    b = rng.integers(-100000, 100000, K).astype(np.int32)
    acc = NC.conv_sum(NC.decode_tensor(x, 8, p), NC.decode_tensor(w, 8, p), stride, pad, groups) + b.astype(np.int64)
    want = int((np.maximum(acc, 0) if relu else np.abs(acc)).max())
    got = B.conv_np_absmax(*planes(B, x, p), *planes(B, w, p), dev(b), stride, pad, groups, relu)
    assert got == want
    if C == 512:
        assert want > 1 << 33
    # all-negative sums under ReLU leave the cleared word
    if relu and C < 512:
        wneg = np.full_like(w, 0xff)
        xpos = np.full_like(x, 0x7f)
        assert B.conv_np_absmax(*planes(B, xpos, p), *planes(B, wneg, p), None, stride, pad, groups, True) == 0


def test_eltwise_np_absmax_and_scale_rule(B):
    rng = np.random.default_rng(3)
    a = rng.integers(0, 256, 100001).astype(np.uint8)
    b = rng.integers(0, 256, 100001).astype(np.uint8)
    for fa, fb, relu in [(5, 5, False), (9, 3, True), (0, 18, False)]:
        _, _, t = NC.eltwise_np(a, (8, 4), fa, b, (8, 4), fb, (8, 4), max(fa, fb), relu)
        want = int((np.maximum(t, 0) if relu else np.abs(t)).max())
        assert B.eltwise_np_absmax(*planes(B, a, 4), fa, *planes(B, b, 4), fb, relu) == want
    for p in (4, 5, 7):
        bm = F.beta_max(8, p)
        for m in [0, 1, bm - 1, bm, bm + 1, 2 * bm, 2 * bm + 1, 12345678, (1 << 36) + 5, bm << 20, (bm << 20) + 1, (1 << 63) + 1]:
            for f_acc in [-3, 0, 7, 20, 40]:
                assert B.np_frac_from_absmax_u64(m, f_acc, 8, p) == NN.frac_from_absmax_int(m, f_acc, 8, p), (m, f_acc, p)


@pytest.mark.parametrize("p", [4, 5, 7])
def test_pool_np_against_oracle(B, p):
    rng = np.random.default_rng(p)
    for shape, mode, k, stride, pad in [((2, 13, 11, 64), "max", 3, 2, 1), ((2, 12, 12, 8), "max", 3, 2, 1), ((1, 9, 9, 5), "max", 3, 2, 1),
                                        ((2, 8, 8, 16), "max", 2, 2, 0), ((1, 7, 7, 6), "max", 3, 1, 1), ((3, 7, 7, 64), "avg", 7, 1, 0), ((5, 7, 7, 2048), "avg", 7, 1, 0), ((2, 5, 5, 12), "avg", 5, 1, 0),
                                        ((1, 8, 8, 10), "avg", 2, 2, 0), ((2, 9, 9, 4), "avg", 3, 3, 0), ((1, 16, 16, 3), "avg", 16, 1, 0)]:
        x = rng.integers(0, 256, shape).astype(np.uint8)
        if mode == "avg":
            x[0, :, :, 0] = 0x7f                                     # a window of largest values: the mean saturates nothing, stays beta_max
            x[0, :, :, 1] = 0xff
        ry, rbeta = NC.pool_np(x, (8, p), mode, k, stride, pad)
        y, yh, yl = B.pool_np(*planes(B, x, p), mode, k, stride, pad, p)
        torch.cuda.synchronize()
        assert np.array_equal(host(y), ry), (shape, mode)
        assert np.array_equal(beta_of((yh, yl)), rbeta)
    # digit planes only, channels a multiple of 16: the kernel that takes the maximum on (h, l) keys without decoding
    for shape in [(2, 13, 11, 64), (3, 57, 58, 32), (1, 8, 8, 16), (2, 112, 112, 64)]:
        x = rng.integers(0, 256, shape).astype(np.uint8)
        _, rbeta = NC.pool_np(x, (8, p), "max", 3, 2, 1)
        _, yh, yl = B.pool_np(*planes(B, x, p), "max", 3, 2, 1, p, want_codes=False)
        assert np.array_equal(beta_of((yh, yl)), rbeta), shape
    # exact ties of the mean (oracle pin: test_average_pool_ties)
    enc = lambda v: F.encode(v, 8, 4)
    if p == 4:
        for vals, want in [((32, 34, 32, 34), 32), ((34, 36, 34, 36), 36), ((2, 0, 0, 0), 0), ((2, 4, 0, 0), 2), ((2, 4, 0, -12), -2)]:
            x = np.array([enc(v) for v in vals], np.uint8).reshape(1, 2, 2, 1)
            _, yh, yl = B.pool_np(*planes(B, x, 4), "avg", 2, 1, 0, 4)
            assert int(beta_of((yh, yl))[0, 0, 0, 0]) == want
    with pytest.raises(B.DfqError):
        B.pool_np(*planes(B, np.zeros((1, 4, 4, 4), np.uint8), p), "avg", 3, 2, 1, p)


@pytest.mark.parametrize("case", [(2, 32, 32, 3, 16, 7, 3), (1, 20, 24, 3, 16, 7, 3), (1, 16, 16, 4, 32, 8, 3), (1, 12, 12, 1, 16, 3, 1), (1, 9, 11, 2, 16, 5, 2)])
def test_packed_first_layer_equals_the_strided_convolution(B, case):
    N, H, W, C, K, R, pad = case
    rng = np.random.default_rng(sum(case))
    x = rng.integers(0, 256, (N, H, W, C)).astype(np.uint8)
    w = rng.integers(0, 256, (K, R, R, C)).astype(np.uint8)
    b = rng.integers(-5000, 5000, K).astype(np.int32)
    ry, rbeta, _ = NC.conv_np(x, (8, 4), w, (8, 4), b, 14, (8, 4), 2, pad, 1, True)
    xh, xl = planes(B, x, 4)
    wh, wl = planes(B, w, 4)
    ph, pl = B.stem_pack_x(xh, R, R, pad), B.stem_pack_x(xl, R, R, pad)
    qh, ql = B.stem_pack_w(wh), B.stem_pack_w(wl)
    P, Q = NC.out_hw(H, W, R, R, 2, pad)
    assert tuple(ph.shape) == (N, P + 3, Q, 64) and tuple(qh.shape) == (K, 4, 1, 64)
    y, yh, yl = B.conv_np(ph, pl, qh, ql, dev(b), 8, 8, 2, 4, 1, 0, 1, True, variant=B.CONV_MFMA)
    torch.cuda.synchronize()
    assert np.array_equal(host(y), ry) and np.array_equal(beta_of((yh, yl)), rbeta)
    assert B.conv_np_absmax(ph, pl, qh, ql, dev(b), 1, 0, 1, True) == B.conv_np_absmax(xh, xl, wh, wl, dev(b), 2, pad, 1, True)


def _compare_all(net, qz, t, oq, ot, p):
    assert qz.frac == oq.frac and qz.w_frac == oq.w_frac
    for name in oq.w:
        assert np.array_equal(host(qz.w_codes[name]), oq.w[name]), name
        K = oq.b[name].shape[0]
        assert np.array_equal(host(qz.b[name])[:K], oq.b[name]), name
    for name, codes in ot.items():
        assert np.array_equal(beta_of(t[name]), NC.decode_tensor(codes, 8, p)), name


@pytest.mark.parametrize("p", [4, 7])
def test_small_resnet_calibration_and_inference(B, p):
    from paper_1805_07941_amd import npnet
    net = wl.resnet50(batch=2, hw=64, classes=24)            # 24 classes: the last layer's filters get zero-padded to 32
    x = net.input_float()
    oq, ot = NN.calibrate(net, x, fmt=(8, p))
    qz, t = npnet.calibrate(net, dev(x), p=p)
    _compare_all(net, qz, t, oq, ot, p)
    x2 = np.ascontiguousarray(np.roll(x, 1, 0) * np.float32(0.8))
    oi = NN.infer(net, oq, x2)
    xd = dev(x2)
    for fuse in (False, True):
        plan = npnet.NpPlan(net, qz, batch=2, fuse=fuse)
        assert (len(plan.fused) >= 12) if fuse else (len(plan.fused) == 0)
        got = host(plan.run(xd))
        torch.cuda.synchronize()
        got = host(plan.logits)
        never_stored = {c.dst for c, _ in plan.fused.values()}
        for name, codes in oi.items():
            if name in never_stored:
                continue
            K = codes.shape[3]
            assert np.array_equal(beta_of(plan.buf[name])[..., :K], NC.decode_tensor(codes, 8, p)), (name, fuse)
        assert np.array_equal(got, NN.logits(net, oq, oi))
    # replayed from a graph, several times with eager work in between
    for rep in range(3):
        plan.logits.zero_()
        out = plan.run_graph(xd)
        torch.cuda.synchronize()
        assert np.array_equal(host(out), NN.logits(net, oq, oi)), rep


def test_resnet50_np84_full_batch(B):
    """The benchmarked configuration: batch 256 at 224 x 224, scales from 8 images, the pass replayed from a graph; two
    whole images - every tensor of the first, the logits of both - against the network oracle, which calibrates for itself."""
    from paper_1805_07941_amd import npnet
    net = wl.resnet50(batch=256)
    x = net.input_float()
    xd = dev(x)
    qz, _ = npnet.calibrate(net, xd[:8].contiguous(), p=4)
    oq, _ = NN.calibrate(net, x[:8], fmt=(8, 4))
    assert qz.frac == oq.frac and qz.w_frac == oq.w_frac
    plan = npnet.NpPlan(net, qz, batch=256)
    plan.run_graph(xd)
    out = plan.run_graph(xd)
    torch.cuda.synchronize()
    pick = [0, 255]
    oi = NN.infer(net, oq, x[pick])
    assert np.array_equal(host(out)[pick], NN.logits(net, oq, oi))
    assert len(plan.fused) == 16
    never_stored = {c.dst for c, _ in plan.fused.values()}
    for name, codes in oi.items():
        if name in never_stored:
            continue
        K = codes.shape[3]
        got = 64 * host(plan.buf[name][0][pick]).astype(np.int64) + host(plan.buf[name][1][pick])
        assert np.array_equal(got[..., :K], NC.decode_tensor(codes, 8, 4)), name
    assert len(np.unique(host(out)[pick])) > 50


ADD_CASES = [
    # N, H, W, C, K, R, stride, pad, mid_shift, relu_mid, d_other (f_other - f_mid), add_shift, relu_out
    (2, 9, 8, 64, 64, 1, 1, 0, 12, False, 0, 1, True),
    (2, 9, 8, 64, 80, 1, 1, 0, 12, False, 2, 3, False),          # channel tail (80 = 64 + 16), other operand finer
    (1, 13, 13, 128, 256, 1, 1, 0, 14, False, -3, 2, True),      # other operand coarser
    (3, 7, 7, 64, 64, 3, 1, 1, 15, True, 0, 0, False),           # ReLU on the layer, none on the sum, no final downscale
    (1, 6, 6, 256, 128, 1, 1, 0, 7, False, 0, 1, True),          # smallest downscale of the 32-bit rounding
    (1, 6, 6, 512, 64, 3, 1, 1, 36, False, 0, 0, True),          # largest
    (1, 5, 5, 64, 64, 1, 1, 0, 12, False, 18, 20, False),        # widest alignment of the layer's result
    (1, 5, 5, 64, 64, 1, 1, 0, 12, False, -18, 5, True),         # and of the other operand
    (1, 5, 5, 64, 64, 1, 1, 0, 12, False, 0, 31, False),         # everything rounds to zero
    (2, 14, 14, 64, 64, 3, 2, 1, 13, False, 1, 2, True),         # strided
    (1, 40, 40, 64, 64, 3, 1, 1, 13, False, 0, 1, True),         # 72-step ring variant is taken from C = 512 only; many tiles here
    (1, 4, 4, 512, 64, 3, 1, 1, 20, False, 0, 1, True),          # three-stage ring (72 steps)
]


@pytest.mark.parametrize("case", ADD_CASES)
def test_conv_np_add_equals_convolution_then_add(B, case):
    import zlib
    N, H, W, C, K, R, stride, pad, mid_shift, relu_mid, d_other, add_shift, relu_out = case
    rng = np.random.default_rng(zlib.crc32(repr(case).encode()))
    sigma = 0.25
    x = gaussian_codes(rng, (N, H, W, C), 4, sigma, relu=True) if mid_shift < 30 else np.full((N, H, W, C), 0x7f, np.uint8)
    w = gaussian_codes(rng, (K, R, R, C), 4, sigma) if mid_shift < 30 else rng.choice(np.array([0x7f, 0xff], np.uint8), (K, R, R, C), p=[0.7, 0.3])
    b = rng.integers(-3000, 3000, K).astype(np.int32)
    P, Q = NC.out_hw(H, W, R, R, stride, pad)
    other = rng.integers(0, 256, (N, P, Q, K)).astype(np.uint8)
    f_mid = 4
    f_x = min(mid_shift, 20)
    f_w = mid_shift + f_mid - f_x
    f_other = f_mid + d_other
    f_y = max(f_mid, f_other) - add_shift
    mid, mid_beta, _ = NC.conv_np(x, (8, 4), w, (8, 4), b, f_x + f_w - f_mid, (8, 4), stride, pad, 1, relu_mid)
    ry, rbeta, _ = NC.eltwise_np(mid, (8, 4), f_mid, other, (8, 4), f_other, (8, 4), f_y, relu_out)
    yh, yl = B.conv_np_add(*planes(B, x, 4), *planes(B, w, 4), dev(b), *planes(B, other, 4), f_x, f_w, f_mid, relu_mid, f_other, f_y, 4, relu_out,
                           stride, pad)
    torch.cuda.synchronize()
    got = beta_of((yh, yl))
    bad = np.argwhere(got != rbeta)
    assert bad.size == 0, (len(bad), bad[:4], got[tuple(bad[0])], rbeta[tuple(bad[0])])
    eh, el = digits_of(rbeta)
    assert np.array_equal(host(yh), eh) and np.array_equal(host(yl), el)
    if add_shift < 20 and mid_shift < 30 and abs(d_other) < 10:
        assert len(np.unique(mid_beta)) > 20 and len(np.unique(rbeta)) > 20


def test_conv_np_add_declines_what_it_does_not_cover(B):
    x = np.zeros((1, 4, 4, 64), np.uint8)
    w = np.zeros((64, 1, 1, 64), np.uint8)
    o = np.zeros((1, 4, 4, 64), np.uint8)
    args = (*planes(B, x, 4), *planes(B, w, 4), None, *planes(B, o, 4))
    # f_x, f_w, f_mid, f_other, f_y: a downscale of the layer's result by 2^2, by 2^37, and a final upscale
    for f_x, f_w, f_mid, f_other, f_y in [(10, 2, 10, 10, 10), (10, 32, 5, 5, 5), (10, 12, 10, 10, 11)]:
        with pytest.raises(B.DfqError) as e:
            B.conv_np_add(*args, f_x, f_w, f_mid, False, f_other, f_y, 4, True)
        assert e.value.status == B.EUNSUPPORTED
    x48 = np.zeros((1, 4, 4, 48), np.uint8)
    w48 = np.zeros((64, 1, 1, 48), np.uint8)
    with pytest.raises(B.DfqError) as e:
        B.conv_np_add(*planes(B, x48, 4), *planes(B, w48, 4), None, *planes(B, o, 4), 10, 12, 10, False, 10, 9, 4, True)
    assert e.value.status == B.EUNSUPPORTED
