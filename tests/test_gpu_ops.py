"""GPU parity: every library call against the CPU oracle, byte for byte, on the same seeded
inputs.  All calls go through the C-ABI (via the ctypes binding)."""
import itertools

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle as orc
import workloads as wl

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


# ---------------------------------------------------------------------------------------- #
def test_quantize_dequantize(B):
    rng = np.random.default_rng(100)
    for n, f in [(1, 0), (3, 4), (4099, 5), (1 << 20, -3), (12345, 12), (777, 32), (64, -32)]:
        x = (rng.standard_normal(n) * 2.0 ** (-f + 5)).astype(np.float32)
        k = min(n, 8)
        x[:k] = np.array([np.nan, np.inf, -np.inf, 0.5 * 2.0 ** -f, 1.5 * 2.0 ** -f, -2.5 * 2.0 ** -f, 1e30, -1e30],
                         np.float32)[:k]
        q = B.quantize(dev(x), f)
        q_ref = orc.quantize(x, f)
        assert np.array_equal(host(q), q_ref), (n, f)
        xd = B.dequantize(q, f)
        assert np.array_equal(host(xd), orc.dequantize(q_ref, f))
    # unaligned views take the narrow path
    x = rng.standard_normal(1001).astype(np.float32)
    xd = dev(x)
    q = torch.empty(1004, dtype=torch.int8, device=DEV)
    B.quantize(xd[1:], 4, out=q[3:1003])
    assert np.array_equal(host(q[3:1003]), orc.quantize(x[1:], 4))
    # empty
    B.quantize(torch.empty(0, dtype=torch.float32, device=DEV), 3)


@pytest.mark.parametrize("n,p", [(8, 4), (8, 3), (8, 2), (8, 7), (8, 6), (8, 5), (6, 0), (7, 3), (6, 3), (5, 1), (4, 0), (2, 1), (2, 0)])
def test_quantize_dequantize_np(B, n, p):
    """The general (n, p) dynamic floating-point codes (Sec. 2.1): conversion kernels against the oracle, code for code -
    random data over the whole range, every midpoint between neighbouring values (ties), every code, specials."""
    import oracle.npfmt as F
    rng = np.random.default_rng(1000 * n + p)
    bm = F.beta_max(n, p)
    reps = sorted(F.decode(c, n, p) for c in range(1 << (n - 1)))
    for frac in (0, 5, -3, 32, -32):
        gamma = bm * 2.0 ** -frac
        x = (rng.standard_normal(1 << 16) * gamma / 3).astype(np.float32)
        x[:4096] = (rng.standard_normal(4096) * 3.0 * 2.0 ** -frac).astype(np.float32)            # subnormal range
        mids = np.array([(a + b) / 2.0 for a, b in zip(reps, reps[1:])], np.float64) * 2.0 ** -frac
        sp = np.array([np.nan, np.inf, -np.inf, 3e38, -3e38, 0.0, -0.0, 1e-45, -1e-45, gamma, -gamma, gamma * 1.01], np.float32)
        x = np.concatenate([x, mids.astype(np.float32), -mids.astype(np.float32), sp, np.array(reps, np.float64).astype(np.float32) * np.float32(2.0 ** -frac)])
        codes_ref, _ = F.quantize(x, n, p, frac)
        q = B.quantize_np(dev(x), n, p, frac)
        assert np.array_equal(host(q), codes_ref.astype(np.uint8)), (n, p, frac)
        assert np.array_equal(host(B.dequantize_np(q, n, p, frac)), F.dequantize(codes_ref, n, p, frac))
        allc = np.arange(1 << n, dtype=np.uint8) if n < 8 else np.arange(256, dtype=np.uint8)
        assert np.array_equal(host(B.dequantize_np(dev(allc), n, p, frac)), F.dequantize(allc, n, p, frac))
    # unaligned views and a ragged tail take the narrow path
    x = (rng.standard_normal(1003) * bm / 4).astype(np.float32)
    q = torch.zeros(1010, dtype=torch.uint8, device=DEV)
    B.quantize_np(dev(x)[1:], n, p, 0, out=q[3:1005])
    assert np.array_equal(host(q[3:1005]), F.quantize(x[1:], n, p, 0)[0].astype(np.uint8))
    B.quantize_np(torch.empty(0, dtype=torch.float32, device=DEV), n, p, 0)
    with pytest.raises(B.DfqError):
        B.quantize_np(dev(x), 9, 4, 0)
    with pytest.raises(B.DfqError):
        B.quantize_np(dev(x), 8, 1, 0)          # six exponent bits


def test_quantize_i32(B):
    rng = np.random.default_rng(101)
    x = (rng.standard_normal(5000) * 0.1).astype(np.float32)
    x[:6] = [np.nan, np.inf, -np.inf, 1e30, -1e30, 0.5]
    for f in (0, 11, 13, 31, 40, 64, -5):
        assert np.array_equal(host(B.quantize_i32(dev(x), f)), orc.quantize_i32(x, f)), f


def test_config0_every_variant(B):
    c = wl.config0()
    y_ref, acc_ref = orc.conv_q(c["x"], c["w"], c["b"], c["f_in"], c["f_w"], c["f_out"], c["stride"], c["pad"],
                                c["groups"], c["relu"], want_acc=True)
    ran = []
    for variant in (B.CONV_AUTO, B.CONV_DIRECT, B.CONV_MFMA):
        try:
            y, acc = B.conv_q(dev(c["x"]), dev(c["w"]), dev(c["b"]), c["f_in"], c["f_w"], c["f_out"], c["stride"],
                              c["pad"], c["groups"], c["relu"], want_acc=True, variant=variant)
        except B.DfqError as e:
            assert e.status == B.EUNSUPPORTED
            continue
        ran.append(variant)
        assert np.array_equal(host(acc), acc_ref), B.CONV_VARIANT_NAMES[variant]
        assert np.array_equal(host(y), y_ref), B.CONV_VARIANT_NAMES[variant]
    assert B.CONV_AUTO in ran and B.CONV_DIRECT in ran


def _rand_conv(rng, N, H, W, C, K, R, S, groups):
    x = rng.integers(-128, 128, (N, H, W, C)).astype(np.int8)
    w = rng.integers(-128, 128, (K, R, S, C // groups)).astype(np.int8)
    b = rng.integers(-2 ** 20, 2 ** 20, (K,)).astype(np.int32)
    return x, w, b


CONV_SHAPES = [
    # N  H   W   C    K   R  S  st pad groups
    (1, 5, 5, 3, 4, 3, 3, 1, 1, 1),
    (2, 9, 7, 16, 24, 3, 3, 1, 1, 1),
    (2, 9, 7, 16, 24, 3, 3, 2, 1, 1),
    (1, 12, 12, 32, 40, 1, 1, 1, 0, 1),
    (3, 14, 14, 64, 64, 3, 3, 1, 1, 1),
    (2, 14, 14, 64, 128, 1, 1, 2, 0, 1),
    (1, 17, 13, 48, 80, 5, 5, 1, 2, 1),
    (2, 8, 8, 128, 96, 3, 3, 2, 1, 1),
    (1, 7, 7, 512, 200, 1, 1, 1, 0, 1),
    (5, 1, 1, 256, 100, 1, 1, 1, 0, 1),          # fully connected
    (40, 1, 1, 1024, 1000, 1, 1, 1, 0, 1),       # fully connected: the one-wavefront-per-tile kernel
    (1, 20, 20, 3, 32, 3, 3, 2, 1, 1),           # stem-like
    (1, 23, 23, 3, 64, 7, 7, 2, 3, 1),           # stem-like 7x7
    (2, 72, 72, 3, 64, 7, 7, 2, 3, 1),           # stem-like, rows long enough for the row-staging kernel
    (1, 40, 44, 3, 32, 3, 3, 1, 1, 1),           # the same kernel at stride 1, ragged last tile
    (1, 70, 68, 4, 64, 5, 5, 2, 2, 1),           # spans too long for it: direct-load kernel
    (2, 10, 10, 32, 32, 3, 3, 1, 1, 32),         # depthwise
    (2, 11, 9, 64, 64, 3, 3, 2, 1, 64),          # depthwise stride 2
    (1, 9, 9, 24, 24, 3, 3, 1, 1, 24),           # depthwise, C % 16 != 0
    (9, 7, 7, 1024, 1024, 3, 3, 1, 1, 1024),     # depthwise, few pixels and C / 4 = the block size: every lane keeps its own weights
    (9, 7, 7, 2048, 2048, 3, 3, 2, 1, 2048),     # C / 4 twice the block size: the grid in whole sets of channels
    # depthwise with whole blocks of 64 channels: the matrix-core form (patches of 8 x 16 outputs)
    (2, 19, 37, 64, 64, 3, 3, 1, 1, 64),         # ragged patches in both directions
    (1, 16, 16, 128, 128, 3, 3, 1, 1, 128),      # exactly two patch rows, one patch column, two channel blocks
    (2, 21, 35, 128, 128, 3, 3, 2, 1, 128),      # stride 2
    (3, 7, 7, 192, 192, 3, 3, 1, 1, 192),        # image smaller than a patch
    (1, 14, 14, 64, 64, 3, 3, 2, 1, 64),         # stride 2, even size
    (1, 12, 20, 64, 64, 3, 3, 1, 0, 64),         # no padding
    (1, 1, 1, 64, 64, 3, 3, 1, 1, 64),           # one pixel: eight of nine taps are padding
    # stride 1 with at least four patches per workgroup of a full grid: every workgroup streams its patches through two buffers
    (128, 45, 52, 96, 96, 3, 3, 1, 1, 96),       # blocks of 32 channels: 9216 units on 1791 workgroups
    (100, 41, 50, 128, 128, 3, 3, 1, 1, 128),    # two blocks of 64 channels, ragged last patch row and column: 4800 units on 1024
    (400, 30, 40, 64, 64, 3, 3, 1, 0, 64),       # no padding
    (800, 20, 30, 64, 64, 3, 3, 1, 2, 64),       # padding of two: outputs outnumber inputs
    (1, 40, 33, 32, 32, 3, 3, 1, 1, 32),         # 32 channels: two pixels per LDS row
    (2, 21, 35, 96, 96, 3, 3, 2, 1, 96),         # three blocks of 32 channels, stride 2
    (1, 8, 8, 16, 32, 3, 3, 1, 1, 4),            # grouped
    (1, 6, 6, 20, 10, 2, 3, 1, 1, 5),            # grouped, odd kernel
    (2, 19, 17, 128, 128, 3, 3, 1, 1, 32),       # grouped: 32 groups of 4 channels, ragged row blocks
    (2, 19, 17, 128, 256, 3, 3, 2, 1, 16),       # grouped, stride 2, 8 input and 16 output channels per group
    (1, 14, 14, 256, 256, 3, 3, 1, 1, 8),        # grouped, 32 channels per group
    (3, 9, 11, 64, 96, 5, 5, 1, 2, 4),           # grouped 5x5
    (2, 13, 13, 96, 48, 1, 1, 1, 0, 12),         # grouped 1x1
    (1, 12, 10, 24, 36, 7, 7, 2, 3, 3),          # grouped 7x7 stride 2
    (1, 9, 9, 12, 8, 3, 3, 1, 1, 4),             # groups of three channels: direct kernel
    # grouped layers whose groups fill blocks of 64 channels: the matrix-core form (zero-padded block-diagonal weights)
    (2, 19, 17, 128, 128, 3, 3, 2, 1, 16),       # groups of 8, stride 2
    (2, 13, 13, 128, 128, 1, 1, 1, 0, 32),       # 1x1, groups of 4: one step per tile
    (1, 10, 10, 128, 128, 3, 3, 1, 1, 2),        # groups of 64: no padding zeros at all
    (1, 9, 9, 64, 64, 2, 3, 1, 1, 4),            # groups of 16, even kernel height
    (3, 29, 31, 192, 192, 3, 3, 1, 1, 24),       # three channel blocks, ragged last pixel tile
    (1, 33, 31, 16, 16, 3, 3, 1, 0, 1),          # no padding
    (1, 40, 40, 64, 256, 3, 3, 1, 1, 1),         # several tiles in both GEMM dimensions
    (9, 64, 64, 64, 128, 3, 3, 1, 1, 1),         # 144 tiles of 256 x 128: more than half the compute units, so that tile shape
    # unpadded 1x1 stride 1: the input-resident pointwise kernel (several pixel tiles, ragged last one)
    (3, 19, 17, 64, 256, 1, 1, 1, 0, 1),
    (2, 23, 21, 256, 384, 1, 1, 1, 0, 1),
    (2, 30, 30, 128, 64, 1, 1, 1, 0, 1),
    (1, 16, 16, 192, 192, 1, 1, 1, 0, 1),
    (2, 14, 14, 256, 1024, 1, 1, 1, 0, 1),
    (1, 3, 3, 64, 256, 1, 1, 1, 0, 1),           # fewer pixels than one tile
    (1, 10, 10, 128, 1088, 1, 1, 1, 0, 1),       # K a multiple of 64 only and large: one workgroup per CU for LDS
    (1, 9, 9, 512, 128, 1, 1, 1, 0, 1),          # C too large for it: general dense kernel
    # at most 1024 pixels, unpadded 1x1, whole 64-byte steps: one wavefront per 32 x 32 tile, a ring of twelve steps
    (256, 1, 1, 2048, 1000, 1, 1, 1, 0, 1),      # the classifier at full batch: 8 x 32 tiles, channel tail of eight
    (33, 1, 1, 832, 1000, 1, 1, 1, 0, 1),        # a pixel tile with one row; thirteen steps: one refill of the ring
    (5, 1, 1, 64, 72, 1, 1, 1, 0, 1),            # a single step
    (7, 3, 3, 192, 130, 1, 1, 1, 0, 1),          # 63 pixels, channel tail of two
    (2, 16, 32, 768, 96, 1, 1, 1, 0, 1),         # 1024 pixels: 32 x 3 tiles, twelve steps: the ring exactly
    # 3x3 stride 1 pad 1 with whole channel chunks on degenerate images
    (2, 9, 7, 128, 128, 3, 3, 1, 1, 1),          # image rows much shorter than a tile
    (5, 3, 1, 64, 64, 3, 3, 1, 1, 1),            # one column: every pixel is at both borders
    (3, 1, 5, 64, 128, 3, 3, 1, 1, 1),           # one row: kernel rows 0 and 2 are all padding
    (1, 37, 29, 256, 256, 3, 3, 1, 1, 1),        # ragged last tile, four channel chunks
    (2, 30, 33, 192, 384, 3, 3, 1, 1, 1),        # three chunks, three channel tiles
    # K a multiple of 256 and enough pixels for 192 tiles of 256 x 256: the dense kernel's largest tile shape
    (4, 111, 112, 16, 256, 3, 3, 1, 1, 1),       # C % 64 != 0, ragged last pixel tile
    (2, 112, 111, 64, 512, 1, 1, 1, 0, 1),       # two channel tiles, 1x1
    (4, 112, 111, 64, 256, 3, 3, 1, 1, 1),       # 3x3, taps uniform per step
]


@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_q_random_shapes(B, shape):
    N, H, W, C, K, R, S, st, pad, g = shape
    rng = np.random.default_rng(abs(hash(shape)) % (2 ** 31))
    x, w, b = _rand_conv(rng, N, H, W, C, K, R, S, g)
    xd, wd, bd = dev(x), dev(w), dev(b)
    variants = [B.CONV_AUTO, B.CONV_DIRECT, B.CONV_MFMA, B.CONV_DEPTHWISE, B.CONV_SMALLC, B.CONV_POINTWISE, B.CONV_GROUPED]
    first = True
    for f_in, f_w, f_out, relu, bias in [(4, 7, 4, 1, True), (3, 6, 2, 0, True), (2, 2, 4, 0, False), (5, 5, -3, 1, True),
                                         (1, 1, 6, 1, True)]:
        y_ref, acc_ref = orc.conv_q(x, w, b if bias else None, f_in, f_w, f_out, st, pad, g, relu, want_acc=True)
        for v in variants:
            try:
                y, acc = B.conv_q(xd, wd, bd if bias else None, f_in, f_w, f_out, st, pad, g, relu, want_acc=first,
                                  variant=v)
            except B.DfqError as e:
                assert e.status == B.EUNSUPPORTED and v not in (B.CONV_AUTO, B.CONV_DIRECT)
                continue
            if first:
                assert np.array_equal(host(acc), acc_ref), B.CONV_VARIANT_NAMES[v]
            assert np.array_equal(host(y), y_ref), (B.CONV_VARIANT_NAMES[v], f_in, f_w, f_out, relu)
        first = False


@pytest.mark.parametrize("shape", [(3, 19, 17, 64, 256), (2, 23, 21, 256, 384), (2, 30, 30, 128, 64), (2, 14, 14, 256, 1024),
                                   (3, 7, 7, 512, 2048), (5, 21, 19, 320, 256), (40, 14, 14, 1024, 512)],
                         ids=lambda s: "x".join(map(str, s)))
def test_conv_q_add_equals_conv_then_eltwise(B, shape):
    """The fused call against the oracle's convolution followed by the oracle's add, for format
    combinations that put the finer scale on either operand, with and without the ReLUs."""
    N, H, W, C, K = shape
    rng = np.random.default_rng(sum(shape))
    x, w, b = _rand_conv(rng, N, H, W, C, K, 1, 1, 1)
    other = rng.integers(-128, 128, (N, H, W, K)).astype(np.int8)
    xd, wd, bd, od = dev(x), dev(w), dev(b), dev(other)
    ran = 0
    for f_in, f_w, f_mid, relu_mid, f_other, f_out, relu_out in [(4, 7, 4, 0, 5, 3, 1), (3, 6, 2, 0, 1, 0, 1), (5, 5, 3, 1, 3, 2, 0),
                                                              (4, 7, 5, 0, 2, 1, 1), (4, 7, 4, 0, 4, 4, 1)]:
        mid, _ = orc.conv_q(x, w, b, f_in, f_w, f_mid, 1, 0, 1, bool(relu_mid))
        ref, _ = orc.eltwise_q(mid, f_mid, other, f_other, f_out, bool(relu_out))
        got = B.conv_q_add(xd, wd, bd, od, f_in, f_w, f_mid, bool(relu_mid), f_other, f_out, bool(relu_out))
        assert got is not None
        assert np.array_equal(host(got), ref), (f_in, f_w, f_mid, relu_mid, f_other, f_out, relu_out)
        ran += 1
    assert ran == 5


def test_conv_q_add_declines_what_it_does_not_cover(B):
    rng = np.random.default_rng(77)
    x, w, b = _rand_conv(rng, 1, 8, 8, 64, 128, 3, 3, 1)          # 3x3: not a pointwise layer
    other = dev(rng.integers(-128, 128, (1, 8, 8, 128)).astype(np.int8))
    assert B.conv_q_add(dev(x), dev(w), dev(b), other, 4, 7, 4, False, 4, 3, True, 1, 1) is None


def test_conv_q_writes_into_a_channel_slice(B):
    rng = np.random.default_rng(102)
    x, w, b = _rand_conv(rng, 2, 10, 10, 32, 48, 3, 3, 1)
    wide = torch.full((2, 10, 10, 100), 99, dtype=torch.int8, device=DEV)
    y_ref, _ = orc.conv_q(x, w, b, 4, 7, 3, 1, 1, 1, True)
    for v in (B.CONV_AUTO, B.CONV_DIRECT):
        wide.fill_(99)
        B.conv_q(dev(x), dev(w), dev(b), 4, 7, 3, 1, 1, 1, True, out=wide.view(-1)[20:], ldy=100, variant=v)
        got = host(wide)
        assert np.array_equal(got[..., 20:68], y_ref)
        assert np.all(got[..., :20] == 99) and np.all(got[..., 68:] == 99)


def test_fully_connected_into_a_row_slice_of_odd_pitch(B):
    """The kernel for very few pixels writing rows of 1000 channels at a pitch that is not a multiple of 16, from an
    offset that is not one either: whole and partial 16-channel groups, aligned and not."""
    rng = np.random.default_rng(104)
    x, w, b = _rand_conv(rng, 37, 1, 1, 512, 1000, 1, 1, 1)
    wide = torch.full((37, 1, 1, 1012), 99, dtype=torch.int8, device=DEV)
    y_ref, _ = orc.conv_q(x, w, b, 4, 7, -3, 1, 0, 1, False)
    assert (np.abs(y_ref) == 127).mean() < 0.1
    for v in (B.CONV_AUTO, B.CONV_MFMA):
        wide.fill_(99)
        B.conv_q(dev(x), dev(w), dev(b), 4, 7, -3, 1, 0, 1, False, out=wide.view(-1)[7:], ldy=1012, variant=v)
        got = host(wide)
        assert np.array_equal(got[..., 7:1007], y_ref)
        assert np.all(got[..., :7] == 99) and np.all(got[..., 1007:] == 99)


def test_conv_q_shift_extremes(B):
    rng = np.random.default_rng(103)
    x, w, b = _rand_conv(rng, 1, 6, 6, 16, 16, 3, 3, 1)
    for f_in, f_w, f_out in [(0, 0, 0), (0, 0, 5), (-3, -2, 4), (10, 10, -12), (16, 16, -1), (32, 32, -32), (0, 0, 32)]:
        y_ref, _ = orc.conv_q(x, w, b, f_in, f_w, f_out, 1, 1, 1, False)
        for v in (B.CONV_AUTO, B.CONV_DIRECT):
            y, _ = B.conv_q(dev(x), dev(w), dev(b), f_in, f_w, f_out, 1, 1, 1, False, variant=v)
            assert np.array_equal(host(y), y_ref), (f_in, f_w, f_out, v)


def test_eltwise_q(B):
    rng = np.random.default_rng(104)
    for n in (1, 15, 16, 1000, 4096 + 7, 1 << 20):
        a = rng.integers(-128, 128, n).astype(np.int8)
        b = rng.integers(-128, 128, n).astype(np.int8)
        for fa, fb, fy, relu in [(4, 4, 4, 0), (4, 4, 3, 1), (5, 2, 3, 0), (2, 6, 1, 1), (3, 4, 5, 0), (0, 7, -1, 0),
                                 (-3, -1, -4, 1), (10, -12, 0, 0)]:
            y_ref, acc_ref = orc.eltwise_q(a, fa, b, fb, fy, relu, want_acc=True)
            y, acc = B.eltwise_q(dev(a), fa, dev(b), fb, fy, relu, want_acc=True)
            assert np.array_equal(host(y), y_ref) and np.array_equal(host(acc), acc_ref), (n, fa, fb, fy, relu)
            y, _ = B.eltwise_q(dev(a), fa, dev(b), fb, fy, relu)
            assert np.array_equal(host(y), y_ref)
    with pytest.raises(B.DfqError):
        B.eltwise_q(dev(a), 30, dev(b), 0, 0)


def test_concat_q(B):
    rng = np.random.default_rng(105)
    for lead, Cs in [((2, 5, 5), (64, 128, 32, 32)), ((1, 3, 3), (3, 1, 4)), ((1, 7, 7), (4, 8, 12)), ((3, 2, 2), (16,)),
                     ((1, 28, 28), (64, 96, 16, 32, 48, 16, 16, 32))]:
        xs = [rng.integers(-128, 128, lead + (c,)).astype(np.int8) for c in Cs]
        fs = [int(v) for v in rng.integers(2, 7, len(Cs))]
        for fy in (min(fs), min(fs) - 2, max(fs)):
            y = B.concat_q([dev(x) for x in xs], fs, fy)
            assert np.array_equal(host(y), orc.concat_q(xs, fs, fy)), (Cs, fs, fy)


def test_concat_q_into_a_channel_slice(B):
    """A group of branches rescaled into a channel slice of a wider tensor: the slice equals the oracle's concat of
    those branches, everything else is untouched."""
    rng = np.random.default_rng(109)
    for lead, Cs, Ct, off in [((2, 5, 5), (64, 32), 256, 128), ((1, 7, 7), (4, 8), 40, 12), ((3, 2, 2), (3, 5), 21, 7),
                              ((2, 28, 28), (16,), 256, 240)]:
        xs = [rng.integers(-128, 128, lead + (c,)).astype(np.int8) for c in Cs]
        fs = [int(v) for v in rng.integers(2, 7, len(Cs))]
        for fy in (min(fs), min(fs) - 3):
            wide = torch.full(lead + (Ct,), 77, dtype=torch.int8, device=DEV)
            B.concat_q_into([dev(x) for x in xs], fs, fy, wide, off)
            got = host(wide)
            n = sum(Cs)
            assert np.array_equal(got[..., off:off + n], orc.concat_q(xs, fs, fy)), (Cs, fs, fy)
            assert np.all(got[..., :off] == 77) and np.all(got[..., off + n:] == 77)


@pytest.mark.parametrize("mode", ["max", "avg"])
def test_pool_q(B, mode):
    rng = np.random.default_rng(106)
    for (N, H, W, C), (k, st, pad) in itertools.product(
            [(2, 14, 14, 64), (1, 9, 7, 3), (2, 8, 8, 20), (3, 7, 7, 128)],
            [(3, 2, 1), (3, 1, 1), (2, 2, 0), (7, 1, 0), (1, 1, 0), (7, 7, 3)]):
        x = rng.integers(-128, 128, (N, H, W, C)).astype(np.int8)
        for f_in, f_out in [(4, 4), (4, 2), (3, 5), (0, -3)]:
            y = B.pool_q(dev(x), mode, k, st, pad, f_in, f_out)
            assert np.array_equal(host(y), orc.pool_q(x, mode, k, st, pad, f_in, f_out)), (N, H, W, C, k, st, pad, f_in, f_out)


def test_max_pool_3x3_large(B):
    """Enough outputs for the specialized 3x3 max-pool kernel: all-negative data (a window position in the
    padding must never win), borders on every side, strides 1 and 2, every rescale direction."""
    rng = np.random.default_rng(108)
    for (N, H, W, C), (st, pad) in itertools.product([(8, 65, 67, 64), (3, 40, 41, 256)], [(2, 1), (1, 1), (2, 0), (1, 2), (3, 2)]):
        for lo, hi in [(-128, 128), (-128, -100)]:
            x = rng.integers(lo, hi, (N, H, W, C)).astype(np.int8)
            for f_in, f_out in [(4, 4), (4, 2), (3, 5)]:
                y = B.pool_q(dev(x), "max", 3, st, pad, f_in, f_out)
                assert np.array_equal(host(y), orc.pool_q(x, "max", 3, st, pad, f_in, f_out)), (N, H, W, C, st, pad, f_in, f_out)


def test_absmax_and_formats(B):
    rng = np.random.default_rng(107)
    for n in (1, 63, 64, 1000, 1 << 20):
        x = rng.standard_normal(n).astype(np.float32) * 7
        if n > 3:
            x[2] = np.nan
        got = float(host(B.absmax_f32(dev(x)))[0])
        assert got == orc.absmax_f32(x)
        a = rng.integers(-2 ** 31, 2 ** 31, n).astype(np.int32)
        for relu in (0, 1):
            assert B.absmax_i32_value(B.absmax_i32(dev(a), relu)) == orc.absmax_i32(a, relu)
    a = np.array([-2 ** 31, 5], np.int32)
    assert B.absmax_i32_value(B.absmax_i32(dev(a))) == 2 ** 31
    assert B.absmax_i32_value(B.absmax_i32(torch.empty(0, dtype=torch.int32, device=DEV))) == 0


def test_mfma_rate_probe_runs_the_stated_work(B):
    """The measurement aid: with all-ones operands every accumulator grows by 32 per instruction, so the
    word each lane stores is 8 accumulators x 16 registers x 32 x iters; the reported operation count is
    blocks x 8 wavefronts x iters x 8 instructions x 2*32^3."""
    blocks, iters = 3, 5
    ones = torch.ones(1 << 15, dtype=torch.int8, device="cuda:0")
    sink = torch.zeros(blocks * 512, dtype=torch.int32, device="cuda:0")
    from paper_1805_07941_amd import probe
    ops = probe.mfma_rate(ones, ones, sink, blocks, iters)
    assert ops == blocks * 8 * iters * 8 * 2 * 32 ** 3
    assert np.array_equal(host(sink), np.full(blocks * 512, 8 * 16 * 32 * iters, dtype=np.int32))
    # the item-pipeline loop: 16 instructions per step and wavefront on all-ones operands, plus the two operand words the
    # sink adds so that the last reads cannot be dropped (four bytes of ones each: 0x01010101)
    ops = probe.item_loop_rate(ones, ones, sink, blocks, iters)
    assert ops == blocks * 8 * iters * 16 * 2 * 32 ** 3
    assert np.array_equal(host(sink), np.full(blocks * 512, 8 * 16 * 32 * 2 * iters + 2 * 0x01010101, dtype=np.int32))


PC_SHAPES = [
    # N  H   W   C    K   R  S  st pad groups
    (1, 5, 5, 3, 4, 3, 3, 1, 1, 1),              # direct kernel
    (2, 9, 7, 16, 24, 3, 3, 2, 1, 1),            # dense kernel, ragged channel tail
    (3, 14, 14, 64, 64, 3, 3, 1, 1, 1),
    (2, 23, 21, 256, 384, 1, 1, 1, 0, 1),        # pointwise geometry: the dense kernel takes it
    (1, 9, 9, 512, 128, 1, 1, 1, 0, 1),
    (1, 23, 23, 3, 64, 7, 7, 2, 3, 1),           # stem-like
    (2, 72, 72, 3, 64, 7, 7, 2, 3, 1),           # stem-like, row-staging kernel
    (2, 10, 10, 32, 32, 3, 3, 1, 1, 32),         # depthwise
    (2, 11, 9, 64, 64, 3, 3, 2, 1, 64),          # depthwise stride 2
    (1, 8, 8, 16, 32, 3, 3, 1, 1, 4),            # grouped
    (2, 19, 17, 128, 256, 3, 3, 2, 1, 16),       # grouped, stride 2
    (5, 1, 1, 256, 100, 1, 1, 1, 0, 1),          # fully connected
    (40, 1, 1, 1024, 1000, 1, 1, 1, 0, 1),       # fully connected: the one-wavefront-per-tile kernel
    (4, 223, 224, 64, 256, 1, 1, 2, 0, 1),       # enough tiles for the dense kernel's largest tile shape
]


@pytest.mark.parametrize("shape", PC_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_conv_q_per_channel_weight_formats(B, shape):
    """dfq_conv_q_pc against the oracle: every channel rescaled by its own shift (Sec. 3), bytes and
    accumulators identical; equal entries reproduce dfq_conv_q."""
    N, H, W, C, K, R, S, st, pad, g = shape
    rng = np.random.default_rng(abs(hash(("pc",) + shape)) % (2 ** 31))
    x, w, b = _rand_conv(rng, N, H, W, C, K, R, S, g)
    xd, wd, bd = dev(x), dev(w), dev(b)
    for f_in, f_out, relu, lo, hi in [(4, 4, 1, 3, 11), (3, 2, 0, 0, 8), (5, -3, 1, 5, 9), (2, 6, 0, -2, 3)]:
        f_w = rng.integers(lo, hi + 1, K).astype(np.int32)
        y_ref, acc_ref = orc.conv_q(x, w, b, f_in, f_w, f_out, st, pad, g, relu, want_acc=True)
        y, acc = B.conv_q_pc(xd, wd, bd, f_in, dev(f_w), f_out, st, pad, g, relu, want_acc=True)
        assert np.array_equal(host(acc), acc_ref)
        assert np.array_equal(host(y), y_ref), (f_in, f_out, relu)
        y2, _ = B.conv_q_pc(xd, wd, bd, f_in, dev(f_w), f_out, st, pad, g, relu)       # without the accumulator dump
        assert np.array_equal(host(y2), y_ref), (f_in, f_out, relu)
    same = np.full(K, 7, np.int32)
    y_pc, _ = B.conv_q_pc(xd, wd, bd, 4, dev(same), 3, st, pad, g, True)
    y_pl, _ = B.conv_q(xd, wd, bd, 4, 7, 3, st, pad, g, True)
    assert np.array_equal(host(y_pc), host(y_pl))


def test_row_wise_weight_preparation(B):
    """Per-row thresholds and conversions (weights with one format per output channel) against the
    oracle's per-row calls."""
    rng = np.random.default_rng(31)
    wf = (rng.standard_normal((37, 3, 3, 5)) * rng.uniform(0.01, 3.0, (37, 1, 1, 1))).astype(np.float32)
    wf[5] = 0.0
    bf = (rng.standard_normal(37) * 0.3).astype(np.float32)
    gam = host(B.absmax_f32_rows(dev(wf)))
    assert np.array_equal(gam, np.array([orc.absmax_f32(wf[k]) for k in range(37)], np.float32))
    f_w = np.array([orc.frac_from_absmax_f32(float(g)) for g in gam], np.int32)
    assert [B.fmt_from_absmax_f32(float(g)) for g in gam] == f_w.tolist()
    q = host(B.quantize_rows(dev(wf), dev(f_w)))
    assert np.array_equal(q, np.stack([orc.quantize(wf[k], int(f_w[k])) for k in range(37)]))
    for f_in in (-3, 4, 9):
        qb = host(B.quantize_i32_rows(dev(bf), dev(f_w), f_in))
        assert np.array_equal(qb, np.array([orc.quantize_i32(bf[k:k + 1], f_in + int(f_w[k]))[0] for k in range(37)], np.int32))


def test_fold_scale(B):
    """The folding pre-pass (affine layer behind a convolution into its float weights) bit for bit against the oracle."""
    rng = np.random.default_rng(33)
    for shape in [(37, 3, 3, 5), (64, 1, 1, 64), (1000, 2048), (3, 7, 7, 3)]:
        w = (rng.standard_normal(shape) * rng.uniform(0.01, 3.0, (shape[0],) + (1,) * (len(shape) - 1))).astype(np.float32)
        b = (rng.standard_normal(shape[0]) * 0.3).astype(np.float32)
        scale = (rng.random(shape[0]) + 0.5).astype(np.float32)
        shift = (rng.standard_normal(shape[0]) * 0.1).astype(np.float32)
        for bb, sh in [(b, shift), (None, shift), (b, None), (None, None)]:
            w_ref, b_ref = orc.fold_scale(w, bb, scale, sh)
            w_g, b_g = B.fold_scale(dev(w), None if bb is None else dev(bb), dev(scale), None if sh is None else dev(sh))
            assert np.array_equal(host(w_g), w_ref) and np.array_equal(host(b_g), b_ref), (shape, bb is None, sh is None)


def test_absmax_per_channel(B):
    rng = np.random.default_rng(32)
    for shape in [(3, 5, 7, 24), (1, 1, 1, 1000), (2, 9, 9, 3), (1, 300, 300, 16)]:
        a = rng.integers(-2 ** 31, 2 ** 31, shape).astype(np.int32)
        for relu in (False, True):
            got = B.absmax_i32_channels_value(B.absmax_i32_channels(dev(a), relu=relu)).astype(np.int64)
            assert np.array_equal(got, orc.absmax_i32_channels(a, relu=relu)), (shape, relu)


@pytest.mark.parametrize("shape", [(3, 19, 17, 64, 256), (2, 23, 21, 128, 384), (2, 30, 30, 128, 64), (2, 14, 14, 256, 512),
                                   (30, 7, 7, 512, 2048), (9, 14, 14, 256, 1024), (40, 14, 14, 1024, 512)],
                         ids=lambda s: "x".join(map(str, s)))
def test_conv_q_pc_add_equals_the_two_calls(B, shape):
    """The fused per-channel convolution + add against the oracle's two steps, and against the library's own."""
    N, H, W, C, K = shape
    rng = np.random.default_rng(abs(hash(("pcadd",) + shape)) % (2 ** 31))
    x, w, b = _rand_conv(rng, N, H, W, C, K, 1, 1, 1)
    other = rng.integers(-128, 128, (N, H, W, K)).astype(np.int8)
    xd, wd, bd, od = dev(x), dev(w), dev(b), dev(other)
    for f_in, f_mid, relu_mid, f_other, f_out, relu_out, lo, hi in [(4, 4, 0, 5, 3, 1, 4, 10), (3, 2, 1, 2, 2, 0, 1, 7),
                                                                   (5, 6, 0, 3, 1, 1, 6, 12)]:
        f_w = rng.integers(lo, hi + 1, K).astype(np.int32)
        mid, _ = orc.conv_q(x, w, b, f_in, f_w, f_mid, 1, 0, 1, relu_mid)
        ref, _ = orc.eltwise_q(mid, f_mid, other, f_other, f_out, relu_out)
        got = B.conv_q_pc_add(xd, wd, bd, od, f_in, dev(f_w), (lo, hi), f_mid, relu_mid, f_other, f_out, relu_out)
        assert got is not None, "the fused per-channel kernel should cover this call"
        assert np.array_equal(host(got), ref), (f_in, f_mid, f_other, f_out)
        # the unfused per-channel pointwise kernel on the same layer
        y, _ = B.conv_q_pc(xd, wd, bd, f_in, dev(f_w), f_mid, 1, 0, 1, relu_mid, frac_w_range=(lo, hi))
        assert np.array_equal(host(y), mid)
    # shifts outside the lean range are declined, not mis-computed
    f_w = np.full(K, 30, np.int32)
    assert B.conv_q_pc_add(xd, wd, bd, od, 4, dev(f_w), (30, 30), 2, False, 3, 3, True) is None


def test_histogram_and_threshold_search(B):
    """dfq_hist_i32 counts exactly what the oracle's histogram counts; the search on it gives the oracle's threshold."""
    rng = np.random.default_rng(61)
    xs = [np.abs(rng.standard_normal((4, 30, 30, 64)) * 5000).astype(np.int32),
          rng.integers(-2 ** 31, 2 ** 31, (3, 7, 11, 24)).astype(np.int32),
          (rng.standard_normal((2, 56, 56, 256)) * 1e5).astype(np.int32),
          np.zeros((1, 3, 3, 8), np.int32)]
    xs[0][0, 0, 0, 0] = 9_000_000
    for x in xs:
        for relu in (False, True):
            counts, j, m = orc.hist_i32(x, relu=relu)
            gm = B.absmax_i32_value(B.absmax_i32(dev(x), relu=relu))
            assert gm == m and B.hist_shift(gm) == j
            h = host(B.hist_i32(dev(x), j, relu=relu)).view(np.uint32)
            assert np.array_equal(h[:len(counts)].astype(np.uint64), counts) and int(h[len(counts):].sum()) == 0
            assert B.threshold_search(h, j, m)[0] == orc.threshold_search(counts, j, m)[0]


# ---------------------------------------------------------------------------------------- #
# The fused convolution + add at the sizes the benchmark launches it with: many more units
# than workgroups, so every workgroup walks a run of units (second operand fetched one unit
# ahead, input buffers handed over between pixel tiles, stores of earlier epilogues in flight).
def _scaled_pointwise_case(rng, N, H, C, K):
    """int8 tensors of a 1x1 layer whose accumulators have a standard deviation near 2^9 * sqrt(C),
    so that a shift of s = 10 + log2(C)/2 - 3 leaves most outputs unsaturated."""
    x = np.clip(np.rint(rng.standard_normal((N, H, H, C), dtype=np.float32) * 16), -128, 127).astype(np.int8)
    w = np.clip(np.rint(rng.standard_normal((K, 1, 1, C), dtype=np.float32) * 32), -128, 127).astype(np.int8)
    b = rng.integers(-2 ** 12, 2 ** 12, (K,)).astype(np.int32)
    other = np.clip(np.rint(rng.standard_normal((N, H, H, K), dtype=np.float32) * 40), -128, 127).astype(np.int8)
    s = 4 + int(round(np.log2(C) / 2))            # accumulator std ~ 16 * 32 * sqrt(C) = 2^(9 + log2(C)/2) -> codes of std ~ 32
    return x, w, b, other, s


@pytest.mark.parametrize("per_channel", [False, True], ids=["per_layer", "per_channel"])
@pytest.mark.parametrize("shape", [(56, 64, 256), (28, 128, 512), (14, 256, 1024), (7, 512, 2048)], ids=lambda s: "x".join(map(str, s)))
def test_conv_q_add_full_size_sampled(B, shape, per_channel):
    """dfq_conv_q_add / dfq_conv_q_pc_add at batch 256 (the benchmark's launch configuration): 400 sampled outputs
    through the oracle's single-element convolution, its rounding and its add; two whole images; and the whole
    tensor against the library's own unfused pair of calls."""
    H, C, K = shape
    N = 256
    rng = np.random.default_rng(5000 + H)
    x, w, b, other, s = _scaled_pointwise_case(rng, N, H, C, K)
    f_in, f_mid, f_other, f_out, relu_mid, relu_out = 4, 3, 4, 3, False, True
    if per_channel:
        f_w = (f_mid - f_in + s + rng.integers(-1, 2, K)).astype(np.int32)      # shifts s-1 .. s+1 by channel
        shifts = f_in + f_w - f_mid
    else:
        f_w = f_mid - f_in + s
        shifts = np.full(K, s)
    xd, wd, bd, od = dev(x), dev(w), dev(b), dev(other)
    if per_channel:
        fwd = dev(f_w)
        rngw = (int(f_w.min()), int(f_w.max()))
        got = B.conv_q_pc_add(xd, wd, bd, od, f_in, fwd, rngw, f_mid, relu_mid, f_other, f_out, relu_out)
        assert got is not None          # (256 -> 1024 and 512 -> 2048 run in the general dense kernel's fused form)
        mid_g, _ = B.conv_q_pc(xd, wd, bd, f_in, fwd, f_mid, 1, 0, 1, relu_mid, frac_w_range=rngw)
        two, _ = B.eltwise_q(mid_g, f_mid, od, f_other, f_out, relu_out)
        assert torch.equal(got, two)
    else:
        got = B.conv_q_add(xd, wd, bd, od, f_in, f_w, f_mid, relu_mid, f_other, f_out, relu_out)
        assert got is not None
        mid_g, _ = B.conv_q(xd, wd, bd, f_in, f_w, f_mid, 1, 0, 1, relu_mid)
        two, _ = B.eltwise_q(mid_g, f_mid, od, f_other, f_out, relu_out)
        assert torch.equal(got, two)
    got = host(got)
    pts = [(0, 0, 0, 0), (N - 1, H - 1, H - 1, K - 1), (N - 1, 0, H - 1, 0), (0, H - 1, 0, K - 1)]
    pts += [tuple(int(v) for v in (rng.integers(N), rng.integers(H), rng.integers(H), rng.integers(K))) for _ in range(400)]
    mids = np.array([orc.requant8(orc.conv_acc_at(x, w, b, 1, 0, 1, n, p, q, k), int(shifts[k])) for (n, p, q, k) in pts], np.int8)
    oth = np.array([other[pt] for pt in pts], np.int8)
    ref, _ = orc.eltwise_q(mids, f_mid, oth, f_other, f_out, relu_out)
    assert np.array_equal(np.array([got[pt] for pt in pts], np.int8), ref)
    assert np.abs(mids).max() > 16 and (np.abs(mids) == 127).mean() < 0.1        # the rounding is exercised, not the clamp
    for n in (0, N - 1):
        mid, _ = orc.conv_q(x[n:n + 1], w, b, f_in, f_w, f_mid, 1, 0, 1, relu_mid)
        ref, _ = orc.eltwise_q(mid, f_mid, other[n:n + 1], f_other, f_out, relu_out)
        assert np.array_equal(got[n:n + 1], ref), n


@pytest.mark.parametrize("shape", [(3, 19, 17, 64, 256), (2, 23, 21, 256, 384), (2, 30, 30, 128, 64), (2, 14, 14, 256, 1024),
                                   (3, 7, 7, 512, 2048), (5, 21, 19, 320, 256), (40, 14, 14, 1024, 512)],
                         ids=lambda s: "x".join(map(str, s)))
def test_conv_q_add_lazy_small(B, shape):
    """The single-rounding join (accumulator + second operand at the accumulator's scale, one rescale) against its
    oracle, on every kernel form that carries it, for alignment shifts from 0 to 22 and final shifts from 0 to 23."""
    N, H, W, C, K = shape
    rng = np.random.default_rng(sum(shape) + 1)
    x, w, b = _rand_conv(rng, N, H, W, C, K, 1, 1, 1)
    other = rng.integers(-128, 128, (N, H, W, K)).astype(np.int8)
    xd, wd, bd, od = dev(x), dev(w), dev(b), dev(other)
    for f_in, f_w, f_other, f_out, relu_out in [(4, 7, 5, 3, True), (4, 9, 4, 0, False), (3, 6, 9, 2, True), (5, 8, 13, -3, False),
                                                (6, 10, -6, -7, False), (5, 6, 11, 11, True), (7, 16, 3, 0, False)]:
        ref = orc.conv_q_add_lazy(x, w, b, other, f_in, f_w, f_other, f_out, relu=relu_out)
        got = B.conv_q_add_lazy(xd, wd, bd, od, f_in, f_w, f_other, f_out, relu_out)
        assert got is not None
        assert np.array_equal(host(got), ref), (f_in, f_w, f_other, f_out, relu_out)
    with pytest.raises(B.DfqError):
        B.conv_q_add_lazy(xd, wd, bd, od, 2, 2, 5, 0, True)           # second operand finer than the accumulator
    with pytest.raises(B.DfqError):
        B.conv_q_add_lazy(xd, wd, bd, od, 16, 16, 4, 8, True)         # 28 bits coarser
    assert B.conv_q_add_lazy(xd, wd, bd, od, 16, 16, 12, 4, True) is None      # final shift 28: no lean form


@pytest.mark.parametrize("shape", [(56, 64, 256), (28, 128, 512), (14, 256, 1024), (7, 512, 2048)], ids=lambda s: "x".join(map(str, s)))
def test_conv_q_add_lazy_full_size_sampled(B, shape):
    """dfq_conv_q_add_lazy at batch 256 (many units per workgroup): sampled outputs through the oracle's single-element
    convolution and exact integer arithmetic, two whole images through the oracle's own call, and a count of where it
    differs from the two-rounding call (it must, somewhere, and rarely by more than one code)."""
    H, C, K = shape
    N = 256
    rng = np.random.default_rng(6000 + H)
    x, w, b, other, s = _scaled_pointwise_case(rng, N, H, C, K)
    f_in, f_other, f_out, relu_out = 4, 4, 3, True
    f_w = f_out - f_in + s + 1                    # final shift s + 1: the sum of two tensors of similar range
    sb = f_in + f_w - f_other
    xd, wd, bd, od = dev(x), dev(w), dev(b), dev(other)
    got_d = B.conv_q_add_lazy(xd, wd, bd, od, f_in, f_w, f_other, f_out, relu_out)
    assert got_d is not None
    got = host(got_d)
    pts = [(0, 0, 0, 0), (N - 1, H - 1, H - 1, K - 1), (N - 1, 0, H - 1, 0), (0, H - 1, 0, K - 1)]
    pts += [tuple(int(v) for v in (rng.integers(N), rng.integers(H), rng.integers(H), rng.integers(K))) for _ in range(400)]
    for pt in pts:
        n, p, q, k = pt
        t = orc.conv_acc_at(x, w, b, 1, 0, 1, n, p, q, k) + (int(other[pt]) << sb)
        assert int(got[pt]) == orc.requant8(max(t, 0), s + 1), pt
    for n in (0, N - 1):
        ref = orc.conv_q_add_lazy(x[n:n + 1], w, b, other[n:n + 1], f_in, f_w, f_other, f_out, relu=relu_out)
        assert np.array_equal(got[n:n + 1], ref), n
        assert 0.2 < (ref > 0).mean() and (ref == 127).mean() < 0.1
    two = B.conv_q_add(xd, wd, bd, od, f_in, f_w, f_other, False, f_other, f_out, relu_out)
    diff = (got_d.to(torch.int16) - two.to(torch.int16)).abs()
    # (more than one code apart only where the two-rounding form clamps the convolution's own result at +-127 first)
    assert 0.001 < float((diff != 0).float().mean()) < 0.5 and float((diff > 1).float().mean()) < 0.05


def _ties_bias(rng, K, s):
    """Bias values that are exact ties or near-ties of a rounding shift by s, with quotients inside [-127, 127]."""
    t = rng.integers(-120, 121, K).astype(np.int64)
    half = (1 << (s - 1)) if s > 0 else 0
    kind = rng.integers(0, 4, K)
    off = np.where(kind == 0, half, np.where(kind == 1, half - 1, np.where(kind == 2, half + 1, rng.integers(0, max(1 << s, 1), K))))
    v = t * (1 << s) + off
    return np.clip(v, -2 ** 31 + 2 ** 24, 2 ** 31 - 2 ** 24).astype(np.int32)


@pytest.mark.parametrize("s", [0, 1, 2, 14, 21, 22, 23, 24])
def test_lean_epilogue_shift_edges(B, s):
    """The four-instruction rounding of the matrix-core kernels over the whole range it is declared for (shift 0 .. 23)
    and the hand-over to the general rounding at 24, on layers that take the lean epilogue (whole channel tiles, aligned
    rows, no accumulator dump).  The accumulators are dominated by a bias built from ties and near-ties of the shift,
    so the results are spread over [-127, 127] instead of saturating."""
    rng = np.random.default_rng(600 + s)
    cases = [(2, 20, 20, 64, 128, 3, 1, 1, B.CONV_MFMA), (2, 20, 20, 64, 64, 3, 1, 1, B.CONV_MFMA),
             (1, 24, 24, 128, 256, 1, 1, 0, B.CONV_MFMA), (2, 33, 31, 64, 256, 1, 1, 0, B.CONV_POINTWISE),
             (1, 40, 40, 256, 128, 1, 1, 0, B.CONV_POINTWISE), (2, 30, 30, 128, 64, 1, 1, 0, B.CONV_POINTWISE)]
    for (N, H, W, C, K, R, st, pad, variant) in cases:
        x = rng.integers(-3, 4, (N, H, W, C)).astype(np.int8)
        w = rng.integers(-3, 4, (K, R, R, C)).astype(np.int8)
        b = _ties_bias(rng, K, s)
        f_in, f_w = 6, 12
        f_out = f_in + f_w - s
        for relu in (False, True):
            ref, _ = orc.conv_q(x, w, b, f_in, f_w, f_out, st, pad, 1, relu)
            if variant == B.CONV_POINTWISE and s > 23:
                with pytest.raises(B.DfqError):
                    B.conv_q(dev(x), dev(w), dev(b), f_in, f_w, f_out, st, pad, 1, relu, variant=variant)
                continue
            y, _ = B.conv_q(dev(x), dev(w), dev(b), f_in, f_w, f_out, st, pad, 1, relu, variant=variant)
            assert np.array_equal(host(y), ref), (N, H, W, C, K, R, s, relu)
            y, _ = B.conv_q(dev(x), dev(w), dev(b), f_in, f_w, f_out, st, pad, 1, relu)
            assert np.array_equal(host(y), ref), (N, H, W, C, K, R, s, relu, "auto")
            assert (np.abs(ref) == 127).mean() < 0.5
        # one weight format per output channel with shifts from 0 (or s - 3) up to s
        lo = max(0, s - 3)
        sk = rng.integers(lo, s + 1, K)
        sk[:2] = (lo, s)
        f_wk = (f_out - f_in + sk).astype(np.int32)
        bk = np.array([_ties_bias(rng, 1, int(v))[0] for v in sk], np.int32)
        ref, _ = orc.conv_q(x, w, bk, f_in, f_wk, f_out, st, pad, 1, True)
        y, _ = B.conv_q_pc(dev(x), dev(w), dev(bk), f_in, dev(f_wk), f_out, st, pad, 1, True,
                           frac_w_range=(int(f_wk.min()), int(f_wk.max())))
        assert np.array_equal(host(y), ref), (N, H, W, C, K, R, s, "per channel")


@pytest.mark.parametrize("sa,sb,add_shift", [(22, 0, 23), (0, 22, 23), (21, 0, 22), (0, 21, 23), (0, 0, 23), (1, 0, 0), (0, 1, 1),
                                             (0, 0, 0), (0, 0, 1), (0, 0, 2)])
def test_fused_add_alignment_and_shift_edges(B, sa, sb, add_shift):
    """dfq_conv_q_add / dfq_conv_q_pc_add with the alignment shifts of Eq. 10 at their largest (21, 22) and the final
    rounding shift at the end of the lean range (23): against the oracle's convolution followed by its add."""
    rng = np.random.default_rng(700 + 31 * sa + 7 * sb + add_shift)
    N, H, W, C, K = 2, 21, 19, 128, 256
    x, w, b, other, s = _scaled_pointwise_case(rng, N, H, C, K)
    x = x[:, :, :W].copy(); other = other[:, :, :W].copy()
    # channels 0 and 1 saturate at both ends whatever the input, and meet the extreme codes of the other operand:
    # sums of -255 and 254 in the join's accumulator
    b[0], b[1] = -2 ** 30, 2 ** 30
    other[:, ::2, :, 0], other[:, 1::2, :, 0] = -128, 127
    other[:, ::2, :, 1], other[:, 1::2, :, 1] = 127, -128
    F = 22                                   # the finer of the two scales
    f_mid, f_other, f_out = F - sa, F - sb, F - add_shift
    f_in = 4
    f_w = f_mid - f_in + s
    xd, wd, bd, od = dev(x), dev(w), dev(b), dev(other)
    for relu_mid, relu_out in [(False, True), (True, False)]:
        mid, _ = orc.conv_q(x, w, b, f_in, f_w, f_mid, 1, 0, 1, relu_mid)
        ref, _ = orc.eltwise_q(mid, f_mid, other, f_other, f_out, relu_out)
        got = B.conv_q_add(xd, wd, bd, od, f_in, f_w, f_mid, relu_mid, f_other, f_out, relu_out)
        assert got is not None and np.array_equal(host(got), ref), (sa, sb, add_shift, relu_mid, relu_out)
        f_wk = (f_w + rng.integers(-2, 3, K)).astype(np.int32)
        mid, _ = orc.conv_q(x, w, b, f_in, f_wk, f_mid, 1, 0, 1, relu_mid)
        ref, _ = orc.eltwise_q(mid, f_mid, other, f_other, f_out, relu_out)
        got = B.conv_q_pc_add(xd, wd, bd, od, f_in, dev(f_wk), (int(f_wk.min()), int(f_wk.max())), f_mid, relu_mid, f_other,
                              f_out, relu_out)
        assert got is not None and np.array_equal(host(got), ref), (sa, sb, add_shift, relu_mid, relu_out, "per channel")


# ---------------------------------------------------------------------------------------- #
# first layers (3 channels, stride 2) on the strip kernel, alone and with the max-pooling fused
STEM_SHAPES = [
    # N  H    W    K   R  S  pad
    (2, 64, 64, 64, 7, 7, 3),        # two column blocks of the plain kernel, one of the pooling kernel; two strips per image
    (3, 224, 224, 64, 7, 7, 3),      # seven column blocks (plain), four pooled column blocks
    (2, 58, 96, 64, 7, 7, 3),        # 29 output rows: the last step is ragged; no fused pooling for an odd row count
    (2, 60, 96, 64, 7, 7, 3),        # 30 output rows = 15 pooled rows: the last step holds one; two pooled column blocks
    (2, 224, 224, 32, 3, 3, 1),      # 3x3 first layer, 32 channels
    (1, 66, 64, 32, 3, 3, 1),        # 33 output rows
    (1, 68, 72, 32, 3, 3, 1),        # 36 output columns: 18 pooled columns, the second block mostly empty
    (2, 64, 64, 64, 7, 5, 2),        # even padding: taps start at an even input column; 31 output rows
    (5, 32, 32, 64, 3, 7, 3),        # one column block, strips of one or two steps
    (1, 40, 244, 64, 7, 7, 3),       # 61 pooled columns: the widest image the pooling kernel takes
]


@pytest.mark.parametrize("shape", STEM_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_stem_kernel_alone_and_with_max_pool(B, shape):
    N, H, W, K, R, S, pad = shape
    rng = np.random.default_rng(abs(hash(shape)) % (2 ** 31))
    x = rng.integers(-128, 128, (N, H, W, 3)).astype(np.int8)
    w = rng.integers(-128, 128, (K, R, S, 3)).astype(np.int8)
    b = rng.integers(-2 ** 16, 2 ** 16, (K,)).astype(np.int32)
    xd, bd = dev(x), dev(b)
    P, Q = (H + 2 * pad - R) // 2 + 1, (W + 2 * pad - S) // 2 + 1
    fused_expected = P % 2 == 0 and Q % 2 == 0 and Q // 2 <= 61
    # shifts 13, 9, 0 (small weights), 23; with and without ReLU (without it the pooling sees negative values)
    cases = [(4, 7, -2, 1, w, True), (4, 7, 2, 0, w, True), (3, 3, 6, 1, np.sign(w).astype(np.int8), False), (12, 12, 1, 0, w, True)]
    for f_in, f_w, f_out, relu, wv, bias in cases:
        wdv = dev(wv)
        y_ref, _ = orc.conv_q(x, wv, b if bias else None, f_in, f_w, f_out, 2, pad, 1, relu)
        for v in (B.CONV_AUTO, B.CONV_SMALLC):
            y, _ = B.conv_q(xd, wdv, bd if bias else None, f_in, f_w, f_out, 2, pad, 1, relu, variant=v)
            assert np.array_equal(host(y), y_ref), (f_in, f_w, f_out, relu, v)
        p_ref = orc.pool_q(y_ref, "max", 3, 2, 1, f_out, f_out)
        p = B.conv_q_maxpool(xd, wdv, bd if bias else None, f_in, f_w, f_out, 2, pad, relu)
        assert (p is not None) == fused_expected
        if p is not None:
            assert np.array_equal(host(p), p_ref), (f_in, f_w, f_out, relu)


def test_quantize_conv_q_maxpool_equals_the_three_calls(B):
    """Float images in: the conversion of Sec. 3 inside the first layer's kernel, against the oracle's quantize, convolution
    and pooling one after the other; values on ties, beyond the clamp, infinities and NaN included."""
    rng = np.random.default_rng(4321)
    for (N, H, W, K, R, pad), f_in in itertools.product([(3, 224, 224, 64, 7, 3), (2, 60, 96, 64, 7, 3), (2, 64, 64, 32, 3, 1), (2, 224, 224, 32, 3, 1), (1, 60, 96, 32, 7, 3)], [5, 0, -2]):
        x = (rng.standard_normal((N, H, W, 3)) * 2.0 ** (2 - f_in)).astype(np.float32)
        x.reshape(-1)[::7] = np.rint(x.reshape(-1)[::7] * 2.0 ** f_in) * 2.0 ** -f_in + 0.5 * 2.0 ** -f_in      # exact ties
        x.reshape(-1)[5::1001] = np.float32(np.inf)
        x.reshape(-1)[6::1003] = np.float32(-np.inf)
        x.reshape(-1)[7::1009] = np.float32(np.nan)
        x.reshape(-1)[8::1013] = np.float32(1e30)
        w = rng.integers(-128, 128, (K, R, R, 3)).astype(np.int8)
        b = rng.integers(-2 ** 14, 2 ** 14, (K,)).astype(np.int32)
        xq = orc.quantize(x, f_in)
        f_w, f_out = 7, f_in + 7 - 12
        y_ref, _ = orc.conv_q(xq, w, b, f_in, f_w, f_out, 2, pad, 1, True)
        p_ref = orc.pool_q(y_ref, "max", 3, 2, 1, f_out, f_out)
        p = B.conv_q_maxpool(dev(x), dev(w), dev(b), f_in, f_w, f_out, 2, pad, True)
        assert p is not None
        assert np.array_equal(host(p), p_ref), (N, H, W, K, R, f_in)
        # one weight format per output channel (shifts 0 .. 23 over the channels), from codes and from float images
        fw = rng.integers(f_out - f_in, f_out - f_in + 24, K).astype(np.int32)
        fw[:2] = (f_out - f_in, f_out - f_in + 23)
        y_pc, _ = orc.conv_q(xq, w, b, f_in, fw, f_out, 2, pad, 1, True)
        p_pc_ref = orc.pool_q(y_pc, "max", 3, 2, 1, f_out, f_out)
        for xin in (dev(xq), dev(x)):
            p = B.conv_q_maxpool(xin, dev(w), dev(b), f_in, dev(fw), f_out, 2, pad, True, frac_w_range=(int(fw.min()), int(fw.max())))
            assert p is not None
            assert np.array_equal(host(p), p_pc_ref), (N, H, W, K, R, f_in, str(xin.dtype))
        # without the pooling: the library has a kernel for float images at 32 output channels
        y = B.quantize_conv_q(dev(x), dev(w), dev(b), f_in, f_w, f_out, 2, pad, True)
        assert (y is not None) == (K == 32 and (W // 2) % 16 == 0)
        if y is not None:
            assert np.array_equal(host(y), y_ref), (N, H, W, K, R, f_in)
        # a channel whose shift leaves the lean range: no fused kernel
        assert B.conv_q_maxpool(dev(xq), dev(w), dev(b), f_in, dev(fw), f_out, 2, pad, True,
                                frac_w_range=(int(fw.min()), int(fw.max()) + 1)) is None


def test_conv_q_maxpool_declines_what_it_does_not_cover(B):
    rng = np.random.default_rng(77)
    x = dev(rng.integers(-128, 128, (1, 70, 72, 3)).astype(np.int8))        # 35 output rows: the last window would hang over
    w = dev(rng.integers(-128, 128, (64, 7, 7, 3)).astype(np.int8))
    assert B.conv_q_maxpool(x, w, None, 4, 7, 4, 2, 3, True) is None
    x = dev(rng.integers(-128, 128, (1, 64, 64, 3)).astype(np.int8))
    assert B.conv_q_maxpool(x, w, None, 4, 7, 4, 2, 3, True, pool_k=2, pool_stride=2, pool_pad=0) is None   # another pooling
    assert B.conv_q_maxpool(x, w, None, 4, 7, 12, 2, 3, True) is None                                        # shift < 0
