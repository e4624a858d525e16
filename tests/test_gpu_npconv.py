"""GPU parity of the multiply-accumulate on (8, p >= 4) dynamic floating-point codes (Sec. 2.2, Eq. 6-9) against the
CPU oracle: codes and digit planes byte for byte, through the C-ABI."""
import zlib

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle.npfmt as F
import oracle.npconv as NC

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1805_07941_amd import binding
    binding.lib()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.cpu().numpy()


def digits_of(beta):
    """The digit planes the library's kernels exchange: beta = 64 * hi + lo, both of the sign of beta."""
    mag = np.abs(beta)
    sg = np.where(beta < 0, -1, 1)
    return (sg * (mag >> 6)).astype(np.int8), (sg * (mag & 63)).astype(np.int8)


def gaussian_codes(rng, shape, p, sigma_over_max=0.25, relu=False):
    """Codes of (8, p) as a max-abs calibrated tensor would hold them: a normal sample (its negative half cut off when
    it stands for a post-ReLU activation) scaled so that its largest magnitude lands on beta_max."""
    v = rng.standard_normal(shape)
    if relu:
        v = np.maximum(v, 0)
    v = v / np.abs(v).max() * F.beta_max(8, p)
    return F.quantize(v.astype(np.float32), 8, p, 0)[0].astype(np.uint8)


def test_np_digits_every_code(B):
    for p in (4, 5, 6, 7):
        codes = np.arange(256, dtype=np.uint8)
        beta = np.array([F.decode(int(c), 8, p) for c in codes])
        hi, lo = B.np_digits(dev(codes), p)
        eh, el = digits_of(beta)
        assert np.array_equal(host(hi), eh) and np.array_equal(host(lo), el)
        assert np.array_equal(64 * host(hi).astype(np.int64) + host(lo), beta)
        # a long ragged array
        rng = np.random.default_rng(p)
        c2 = rng.integers(0, 256, 100003).astype(np.uint8)
        h2, l2 = B.np_digits(dev(c2), p)
        assert np.array_equal(64 * host(h2).astype(np.int64) + host(l2), NC.decode_tensor(c2, 8, p))
    B.np_digits(torch.empty(0, dtype=torch.uint8, device=DEV), 4)
    with pytest.raises(B.DfqError):
        B.np_digits(dev(np.zeros(4, np.uint8)), 3)


def run_both(B, x, px, w, pw, b, f_x, f_w, f_y, p_y, stride, pad, groups, relu, variant):
    xh, xl = B.np_digits(dev(x), px)
    wh, wl = B.np_digits(dev(w), pw)
    y, yh, yl = B.conv_np(xh, xl, wh, wl, None if b is None else dev(b.astype(np.int32)), f_x, f_w, f_y, p_y, stride, pad,
                          groups, relu, variant=variant)
    torch.cuda.synchronize()
    ry, rbeta, _ = NC.conv_np(x, (8, px), w, (8, pw), b, f_x + f_w - f_y, (8, p_y), stride, pad, groups, relu)
    eh, el = digits_of(rbeta)
    gy, gh, gl = host(y), host(yh), host(yl)
    bad = np.argwhere(gy != ry)
    assert bad.size == 0, (len(bad), bad[:5], gy[tuple(bad[0])], ry[tuple(bad[0])])
    assert np.array_equal(gh, eh) and np.array_equal(gl, el)
    return ry, rbeta


# N, H, W, C, K, R, S, stride, pad, px, pw, p_y, shift, relu, data
MFMA_CASES = [
    (2, 9, 7, 64, 32, 3, 3, 1, 1, 4, 4, 4, 14, False, "gauss"),          # one ragged tile of 256 x 64
    (3, 12, 11, 128, 80, 3, 3, 1, 1, 4, 4, 4, 15, True, "gauss"),        # four pixel tiles of 128, ragged channel tile
    (1, 17, 15, 64, 64, 1, 1, 1, 0, 4, 4, 4, 11, False, "uniform"),      # 1 x 1, K = 64
    (2, 16, 16, 192, 144, 3, 3, 2, 1, 4, 5, 5, 17, True, "uniform"),     # stride 2, two channel tiles, mixed formats
    (1, 8, 8, 512, 32, 3, 3, 1, 1, 4, 4, 4, 25, False, "extreme"),       # 4608 terms at the extremes: sums beyond 32 bits
    (2, 11, 13, 64, 48, 5, 5, 2, 2, 4, 4, 6, 18, False, "uniform"),      # 5 x 5, stride 2
    (1, 6, 20, 128, 256, 1, 7, 1, 3, 5, 4, 4, 16, True, "gauss"),        # 1 x 7 kernel, two channel tiles
    (5, 7, 7, 256, 128, 3, 3, 1, 1, 4, 4, 7, 20, False, "uniform"),      # int8 output
    (1, 9, 9, 64, 16, 3, 3, 1, 0, 4, 4, 4, 0, False, "gauss"),           # no padding, shift 0: saturation everywhere
    (1, 5, 5, 64, 16, 3, 3, 1, 1, 4, 4, 4, -3, False, "small"),          # upscale
    (1, 5, 5, 64, 16, 3, 3, 1, 1, 4, 4, 4, 30, False, "gauss"),          # everything among the subnormals / zero
    (2, 9, 7, 64, 32, 3, 3, 1, 1, 4, 4, 4, 7, False, "small"),           # the smallest shift of the 32-bit epilogue
    (2, 9, 7, 64, 32, 3, 3, 1, 1, 4, 4, 4, 6, True, "small"),            # ... and the one below it
    (1, 6, 6, 128, 48, 3, 3, 1, 1, 4, 4, 5, 36, False, "extreme"),       # the largest, and the one above it
    (1, 6, 6, 128, 48, 3, 3, 1, 1, 4, 4, 5, 37, True, "extreme"),
]


@pytest.mark.parametrize("case", MFMA_CASES)
def test_conv_np_against_oracle(B, case):
    N, H, W, C, K, R, S, stride, pad, px, pw, p_y, shift, relu, data = case
    rng = np.random.default_rng(zlib.crc32(repr(case).encode()))
    if data == "gauss":
        x = gaussian_codes(rng, (N, H, W, C), px, relu=True)
        w = gaussian_codes(rng, (K, R, S, C), pw)
    elif data == "uniform":
        x = rng.integers(0, 256, (N, H, W, C)).astype(np.uint8)
        w = rng.integers(0, 256, (K, R, S, C)).astype(np.uint8)
    elif data == "small":
        x = rng.integers(0, 4, (N, H, W, C)).astype(np.uint8)
        w = (rng.integers(0, 3, (K, R, S, C)) | (rng.integers(0, 2, (K, R, S, C)) << 7)).astype(np.uint8)
    else:
        # every code at +-beta_max, signs arranged so that some outputs add everything up with one sign
        x = np.full((N, H, W, C), 0x7f, np.uint8)
        w = np.where(rng.integers(0, 2, (K, 1, 1, 1)) == 1, 0x7f, 0xff).astype(np.uint8) * np.ones((K, R, S, C), np.uint8)
        w[K // 2:] = np.where(rng.integers(0, 2, (K - K // 2, R, S, C)) == 1, 0x7f, 0xff).astype(np.uint8)
    b = rng.integers(-(1 << 20), 1 << 20, K)
    f_x, f_w = 9, min(shift - 9 + 3, 32)
    f_y = f_x + f_w - shift
    for variant in (B.CONV_MFMA, B.CONV_DIRECT):
        ry, rbeta = run_both(B, x, px, w, pw, b, f_x, f_w, f_y, p_y, stride, pad, 1, relu, variant)
    if data == "extreme":
        _, _, acc = NC.conv_np(x, (8, px), w, (8, pw), b, shift, (8, p_y), stride, pad, 1, relu)
        assert np.abs(acc).max() > 1 << 32                                   # the case means what it says
    if data in ("gauss", "uniform") and shift not in (0, 30):
        mags = np.abs(rbeta)
        assert (mags > 0).mean() > 0.2 and (mags == F.beta_max(8, p_y)).mean() < 0.5       # neither all zero nor all saturated
    # without bias, codes only / digits only
    xh, xl = B.np_digits(dev(x), px)
    wh, wl = B.np_digits(dev(w), pw)
    y1, _, _ = B.conv_np(xh, xl, wh, wl, None, f_x, f_w, f_y, p_y, stride, pad, 1, relu, want_digits=False)
    _, yh2, yl2 = B.conv_np(xh, xl, wh, wl, None, f_x, f_w, f_y, p_y, stride, pad, 1, relu, want_codes=False)
    ry0, rb0, _ = NC.conv_np(x, (8, px), w, (8, pw), None, shift, (8, p_y), stride, pad, 1, relu)
    assert np.array_equal(host(y1), ry0)
    eh, el = digits_of(rb0)
    assert np.array_equal(host(yh2), eh) and np.array_equal(host(yl2), el)


@pytest.mark.parametrize("shift,p_y,relu", [(7, 4, False), (8, 4, True), (13, 5, False), (20, 4, False), (31, 4, True), (36, 4, False),
                                             (37, 4, False), (6, 4, False), (3, 6, True), (0, 4, False), (-2, 4, False), (16, 7, False)])
def test_conv_np_rounding_on_chosen_accumulators(B, shift, p_y, relu):
    """Accumulator values placed on and next to every tie and every representable value of the output format (and beyond
    saturation), up to 2^33 in magnitude: 1 x 1 convolution over 1024 channels of codes +-beta_max, n of them nonzero
    in channel k's weights, plus a bias that fills in the rest: acc = +-1984^2 * n + bias."""
    rng = np.random.default_rng(1000 + shift)
    reps = sorted(F.decode(c, 8, p_y) for c in range(128))
    grid = set()
    for a_, b_ in zip(reps, reps[1:]):
        for num in (2 * a_, a_ + b_, 2 * b_):                       # value, midpoint, next value - all times two
            v2 = num * 2 ** shift if shift >= 0 else None
            if v2 is None:
                if (num % (2 ** (1 - shift))) == 0:
                    base = [num // (2 ** (1 - shift))]
                else:
                    base = [num // (2 ** (1 - shift)), num // (2 ** (1 - shift)) + 1]
            elif v2 % 2 == 0:
                base = [v2 // 2]
            else:
                base = [v2 // 2, v2 // 2 + 1]
            for v in base:
                grid.update((v - 1, v, v + 1, -v, -v - 1, -v + 1))
    top = reps[-1] * 2 ** max(shift, 0)
    grid.update(int(top * f) for f in (1.001, 1.02, 1.5, 3.0))
    C, cap = 1024, 1984 * 1984 * 1024 + (1 << 31) - 1
    vals = sorted(v for v in grid if abs(v) <= cap)
    vals += [int(v) for v in rng.integers(-cap, cap, 500)]
    K = (len(vals) + 15) // 16 * 16
    vals += [0] * (K - len(vals))
    vals = np.array(vals, dtype=np.int64)
    n1 = np.clip(np.rint(np.abs(vals) / 1984.0 ** 2), 0, C).astype(np.int64)
    sg = np.where(vals < 0, -1, 1)
    bias = vals - sg * n1 * 1984 * 1984
    assert np.abs(bias).max() < 1 << 31
    w = np.zeros((K, 1, 1, C), np.uint8)
    for k in range(K):
        w[k, 0, 0, :n1[k]] = 0x7f if sg[k] > 0 else 0xff
    x = np.full((2, 1, 3, C), 0x7f, np.uint8)
    f_x = 9
    f_w = min(shift - 9 + 3, 32)
    f_y = f_x + f_w - shift
    for variant in (B.CONV_MFMA, B.CONV_DIRECT):
        _, _ = run_both(B, x, 4, w, 4, bias, f_x, f_w, f_y, p_y, 1, 0, 1, relu, variant)
    _, _, acc = NC.conv_np(x, (8, 4), w, (8, 4), bias, shift, (8, p_y), 1, 0, 1, relu)
    assert np.array_equal(acc[0, 0, 0], vals)


DIRECT_CASES = [
    (2, 9, 8, 3, 16, 3, 3, 2, 1, 1),        # first layer: C = 3
    (1, 7, 7, 32, 32, 3, 3, 1, 1, 32),      # depthwise
    (2, 6, 6, 24, 36, 3, 3, 1, 1, 4),       # grouped
    (1, 10, 10, 40, 24, 1, 1, 1, 0, 1),     # C not a multiple of 64
    (1, 6, 6, 64, 24, 3, 3, 1, 1, 1),       # K not a multiple of 16
]


@pytest.mark.parametrize("case", DIRECT_CASES)
def test_conv_np_direct_geometries(B, case):
    N, H, W, C, K, R, S, stride, pad, groups = case
    rng = np.random.default_rng(zlib.crc32(repr(case).encode()))
    x = rng.integers(0, 256, (N, H, W, C)).astype(np.uint8)
    w = rng.integers(0, 256, (K, R, S, C // groups)).astype(np.uint8)
    b = rng.integers(-50000, 50000, K)
    shift = int(np.ceil(np.log2(R * S * (C // groups)))) // 2 + 12
    run_both(B, x, 4, w, 4, b, 10, shift - 10 + 2, 2, 4, stride, pad, groups, True, B.CONV_AUTO)
    xh, xl = B.np_digits(dev(x), 4)
    wh, wl = B.np_digits(dev(w), 4)
    with pytest.raises(B.DfqError) as e:
        B.conv_np(xh, xl, wh, wl, None, 10, 5, 2, 4, stride, pad, groups, variant=B.CONV_MFMA)
    assert e.value.status == B.EUNSUPPORTED


def test_three_layers_through_digit_planes(B):
    """A small stack, the planes of one layer feeding the next; the oracle runs the same stack on codes."""
    rng = np.random.default_rng(77)
    N, H, W = 4, 14, 14
    chans = [64, 128, 128, 64]
    xf = rng.standard_normal((N, H, W, chans[0])).astype(np.float32)
    f_x = 9                                                  # 1984 / 2^9 = 3.9: the sample's range
    x_codes, _ = F.quantize(xf, 8, 4, f_x)
    x_codes = x_codes.astype(np.uint8)
    q = B.quantize_np(dev(xf), 8, 4, f_x)
    assert np.array_equal(host(q), x_codes)
    xh, xl = B.np_digits(q, 4)
    ref = x_codes
    f_in = f_x
    for i in range(3):
        C, K = chans[i], chans[i + 1]
        R = 3 if i != 1 else 1
        wf = (rng.standard_normal((K, R, R, C)) * np.sqrt(2.0 / (R * R * C))).astype(np.float32)
        f_w = int(np.floor(np.log2(1984 / np.abs(wf).max())))
        w_codes = F.quantize(wf, 8, 4, f_w)[0].astype(np.uint8)
        b = np.rint(rng.standard_normal(K) * 0.05 * 2.0 ** (f_in + f_w)).astype(np.int64)
        f_y = 8
        wh, wl = B.np_digits(B.quantize_np(dev(wf), 8, 4, f_w), 4)
        y, xh, xl = B.conv_np(xh, xl, wh, wl, dev(b.astype(np.int32)), f_in, f_w, f_y, 4, 1, R // 2, 1, relu=(i < 2))
        ref, rbeta, _ = NC.conv_np(ref, (8, 4), w_codes, (8, 4), b, f_in + f_w - f_y, (8, 4), 1, R // 2, 1, relu=(i < 2))
        assert np.array_equal(host(y), ref), i
        assert (np.abs(rbeta) > 0).mean() > 0.3
        f_in = f_y
    out = B.dequantize_np(y, 8, 4, f_in)
    assert np.array_equal(host(out), F.dequantize(ref, 8, 4, f_in))


@pytest.mark.parametrize("shape", [(256, 56, 64, 64, 3), (256, 7, 512, 512, 3), (256, 14, 256, 1024, 1)])
def test_conv_np_full_size_sampled(B, shape):
    """The layer shapes and batch of the benchmark, in the launch configuration that is timed: sampled outputs against
    plain integer loops, a few whole pixels' channel vectors, and the planes against the codes everywhere."""
    N, H, C, K, R = shape
    rng = np.random.default_rng(H * 1000 + C)
    g = torch.Generator(device="cpu").manual_seed(H * 7 + C)
    x = torch.randint(0, 256, (N, H, H, C), dtype=torch.uint8, generator=g)
    x = torch.where(torch.rand(x.shape, generator=g) < 0.5, torch.zeros_like(x), x & 0x7f)       # post-ReLU: half zeros, no negatives
    w = gaussian_codes(rng, (K, R, R, C), 4)
    b = rng.integers(-(1 << 16), 1 << 16, K)
    shift = 10 + int(round(0.5 * np.log2(R * R * C))) + 5
    xh, xl = B.np_digits(x.to(DEV), 4)
    wh, wl = B.np_digits(dev(w), 4)
    y, yh, yl = B.conv_np(xh, xl, wh, wl, dev(b.astype(np.int32)), shift, 0, 0, 4, 1, R // 2, 1, relu=True)
    torch.cuda.synchronize()
    gy = host(y)
    xn = x.numpy()
    bx = NC.decode_tensor(xn, 8, 4)
    bw = NC.decode_tensor(w, 8, 4)
    P = H
    picks = [(0, 0, 0, 0), (N - 1, P - 1, P - 1, K - 1), (N - 1, 0, P - 1, 0), (N // 2, P // 2, 0, K // 2)]
    picks += [(int(rng.integers(N)), int(rng.integers(P)), int(rng.integers(P)), int(rng.integers(K))) for _ in range(300)]
    nz = 0
    for (n, p, q, k) in picks:
        acc = NC.conv_sum_at(bx, bw, b, 1, R // 2, 1, n, p, q, k)
        want = int(F.round_to_beta(np.ldexp(np.float64(max(acc, 0)), -shift), 8, 4))
        assert F.decode(int(gy[n, p, q, k]), 8, 4) == want, (n, p, q, k, acc)
        nz += want != 0
    assert nz > 60
    # whole channel vectors of a few pixels by the oracle's own convolution on a cut-out
    for (n, p, q) in [(0, 0, 0), (N - 1, P - 1, P - 1), (N // 3, P // 2, P // 3)]:
        lo_p, hi_p = max(p - R // 2, 0), min(p + R // 2, H - 1)
        lo_q, hi_q = max(q - R // 2, 0), min(q + R // 2, H - 1)
        patch = np.zeros((1, R, R, C), np.uint8)
        patch[0, lo_p - (p - R // 2):hi_p - (p - R // 2) + 1, lo_q - (q - R // 2):hi_q - (q - R // 2) + 1] = xn[n, lo_p:hi_p + 1, lo_q:hi_q + 1]
        ry, _, _ = NC.conv_np(patch, (8, 4), w, (8, 4), b, shift, (8, 4), 1, 0, 1, relu=True)
        assert np.array_equal(gy[n, p, q], ry[0, 0, 0])
    # planes and codes agree everywhere (a property that holds at any size)
    beta = torch.from_numpy(NC.decode_tensor(np.arange(256, dtype=np.uint8), 8, 4)).to(DEV)[y.long()]
    assert torch.equal(64 * yh.long() + yl.long(), beta)
    assert bool(((yh.long() * yl.long()) >= 0).all())


ELT_CASES = [
    # p_a, f_a, p_b, f_b, p_y, f_y, relu, n
    (4, 9, 4, 9, 4, 8, False, 100003),
    (4, 9, 4, 6, 4, 5, True, 65536),
    (4, 3, 5, 12, 4, 2, False, 4099),
    (5, 7, 4, 7, 6, 9, False, 777),            # finer result: exact, saturating where it does not fit
    (4, 5, 4, 5, 4, 12, True, 5000),           # upscale by 2^7
    (4, 18, 4, 0, 4, 0, False, 33000),         # the widest alignment allowed
    (4, 0, 4, 18, 5, 31 - 13, False, 33000),
    (4, 10, 4, 10, 4, -21, False, 3000),       # final factor 2^-31: everything rounds to zero
    (4, 4, 4, 4, 4, 20, False, 3000),          # final factor 2^16: saturates unless zero
    (7, 4, 6, 5, 7, 3, True, 20001),           # the int8 members
    (4, 6, 4, 6, 7, 0, False, 20001),
    (4, 8, 4, 8, 4, 7, False, 15),             # shorter than one vector
    (4, 8, 4, 8, 4, 7, False, 1),
]


@pytest.mark.parametrize("case", ELT_CASES)
def test_eltwise_np_against_oracle(B, case):
    p_a, f_a, p_b, f_b, p_y, f_y, relu, n = case
    rng = np.random.default_rng(zlib.crc32(repr(case).encode()))
    a = rng.integers(0, 256, n).astype(np.uint8)
    b = rng.integers(0, 256, n).astype(np.uint8)
    a[: min(n, 8)] = [0x7f, 0xff, 0x00, 0x80, 0x7f, 0xff, 0x01, 0x81][: min(n, 8)]
    b[: min(n, 8)] = [0x7f, 0xff, 0x7f, 0x00, 0xff, 0x7f, 0x81, 0x01][: min(n, 8)]
    ah, al = B.np_digits(dev(a), p_a)
    bh, bl = B.np_digits(dev(b), p_b)
    y, yh, yl = B.eltwise_np(ah, al, f_a, bh, bl, f_b, f_y, p_y, relu)
    torch.cuda.synchronize()
    ry, rbeta, _ = NC.eltwise_np(a, (8, p_a), f_a, b, (8, p_b), f_b, (8, p_y), f_y, relu)
    eh, el = digits_of(rbeta)
    bad = np.flatnonzero(host(y) != ry)
    assert bad.size == 0, (len(bad), bad[:5], host(y)[bad[:5]], ry[bad[:5]])
    assert np.array_equal(host(yh), eh) and np.array_equal(host(yl), el)
    # one kind of output only, and operands that do not start on a 16-byte boundary
    if n > 40:
        y2, _, _ = B.eltwise_np(ah[3:], al[3:], f_a, bh[3:], bl[3:], f_b, f_y, p_y, relu, want_digits=False)
        _, yh3, yl3 = B.eltwise_np(ah, al, f_a, bh, bl, f_b, f_y, p_y, relu, want_codes=False)
        torch.cuda.synchronize()
        assert np.array_equal(host(y2), ry[3:]) and np.array_equal(host(yh3), eh) and np.array_equal(host(yl3), el)


def test_eltwise_np_every_pair_of_codes(B):
    """All 256 x 256 pairs of (8, 4) codes, on a few scale settings: every binade boundary and every tie there is."""
    a = np.repeat(np.arange(256, dtype=np.uint8), 256)
    b = np.tile(np.arange(256, dtype=np.uint8), 256)
    ah, al = B.np_digits(dev(a), 4)
    bh, bl = B.np_digits(dev(b), 4)
    for f_a, f_b, f_y, p_y, relu in [(5, 5, 4, 4, False), (5, 5, 5, 4, False), (6, 4, 3, 4, True), (4, 7, 2, 5, False), (3, 3, 1, 7, False)]:
        y, yh, yl = B.eltwise_np(ah, al, f_a, bh, bl, f_b, f_y, p_y, relu)
        torch.cuda.synchronize()
        ry, rbeta, _ = NC.eltwise_np(a, (8, 4), f_a, b, (8, 4), f_b, (8, p_y), f_y, relu)
        assert np.array_equal(host(y), ry)
        assert np.array_equal(64 * host(yh).astype(np.int64) + host(yl), rbeta)


def test_residual_join_through_digit_planes(B):
    """conv -> add with an identity branch -> conv, every tensor staying in digit planes between the kernels."""
    rng = np.random.default_rng(5)
    N, H, W, C = 2, 14, 14, 64
    x = gaussian_codes(rng, (N, H, W, C), 4, relu=True)
    w1 = gaussian_codes(rng, (C, 3, 3, C), 4)
    w2 = gaussian_codes(rng, (C, 1, 1, C), 4)
    f_x, f_w, f_1, f_j, f_2 = 8, 12, 5, 5, 3
    xh, xl = B.np_digits(dev(x), 4)
    w1h, w1l = B.np_digits(dev(w1), 4)
    w2h, w2l = B.np_digits(dev(w2), 4)
    _, h1, l1 = B.conv_np(xh, xl, w1h, w1l, None, f_x, f_w, f_1, 4, 1, 1, 1, False, want_codes=False)
    _, hj, lj = B.eltwise_np(h1, l1, f_1, xh, xl, f_x, f_j, 4, True, want_codes=False)
    y, _, _ = B.conv_np(hj, lj, w2h, w2l, None, f_j, f_w, f_2, 4, 1, 0, 1, True, want_digits=False)
    torch.cuda.synchronize()
    r1, _, _ = NC.conv_np(x, (8, 4), w1, (8, 4), None, f_x + f_w - f_1, (8, 4), 1, 1, 1, False)
    rj, _, _ = NC.eltwise_np(r1, (8, 4), f_1, x, (8, 4), f_x, (8, 4), f_j, True)
    ry, _, _ = NC.conv_np(rj, (8, 4), w2, (8, 4), None, f_j + f_w - f_2, (8, 4), 1, 0, 1, True)
    assert np.array_equal(host(y), ry)
    assert len(np.unique(ry)) > 20
