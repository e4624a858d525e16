"""Pins of the network-level oracle on (n, p) codes: the member (8, 7) - whose codes are the int8 integers - must reproduce
the int8 network oracle (pinned on its own) tensor for tensor, scales included; the scale rule against exact rationals;
pooling against fractions and the enumerated code set; structural checks on an (8, 4) run."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import oracle.net as onet
import oracle.npconv as NC
import oracle.npfmt as F
import oracle.npnet as NN
import workloads as wl

from test_oracle_npconv import _nearest_by_enumeration


def test_scale_rule_against_fractions():
    for n, p in [(8, 4), (8, 5), (8, 7)]:
        bm = F.beta_max(n, p)
        for m in [0, 1, bm - 1, bm, bm + 1, 2 * bm, 2 * bm + 1, 12345678, (1 << 36) + 5, bm << 20, (bm << 20) + 1]:
            for f_acc in [-3, 0, 7, 20, 40]:
                f = NN.frac_from_absmax_int(m, f_acc, n, p)
                assert -32 <= f <= min(f_acc, 32)
                g = Fraction(m) / Fraction(2) ** f_acc
                assert g * Fraction(2) ** f <= bm or f == -32
                if f < min(f_acc, 32):
                    assert g * Fraction(2) ** (f + 1) > bm                      # one step finer would clip
    # where the threshold is a float32, and the cap does not bind, the float rule says the same
    for m, f_acc in [(1984, 0), (1985, 0), (3000, 4), (100000, 10), (31, 2)]:
        f = NN.frac_from_absmax_int(m, f_acc, 8, 4)
        if f < f_acc:
            assert f == F.frac_from_absmax(m / 2.0 ** f_acc, 8, 4)
    assert [NN.frac_from_absmax_int(m, 5, 8, 7) for m in (0, 127, 128, 254, 255, 1 << 20)] == \
           [oracle.frac_from_absmax_i32(m, 5) for m in (0, 127, 128, 254, 255, 1 << 20)]


@pytest.mark.parametrize("fmt", [(8, 4), (8, 5), (8, 7)])
def test_pool_np_against_fractions_and_enumeration(fmt):
    rng = np.random.default_rng(fmt[1])
    x = rng.integers(0, 256, (2, 7, 6, 3)).astype(np.uint8)
    beta = NC.decode_tensor(x, *fmt)
    for k, stride, pad in [(3, 2, 1), (2, 2, 0), (3, 1, 1)]:
        y, by = NC.pool_np(x, fmt, "max", k, stride, pad)
        P, Q = NC.out_hw(7, 6, k, k, stride, pad)
        for n in range(2):
            for p in range(P):
                for q in range(Q):
                    for c in range(3):
                        vals = [int(beta[n, ih, iw, c]) for ih in range(p * stride - pad, p * stride - pad + k)
                                for iw in range(q * stride - pad, q * stride - pad + k) if 0 <= ih < 7 and 0 <= iw < 6]
                        assert by[n, p, q, c] == max(vals)
                        assert F.decode(int(y[n, p, q, c]), *fmt) == max(vals) and y[n, p, q, c] != 0x80
    for k, stride in [(7, 1), (3, 2), (2, 1), (6, 1)]:
        H = W = 7 if k != 6 else 6
        xs = x[:, :H, :W, :] if k != 6 else x[:, :6, :6, :]
        y, by = NC.pool_np(xs, fmt, "avg", k, stride, 0)
        bs = NC.decode_tensor(xs, *fmt)
        P, Q = NC.out_hw(xs.shape[1], xs.shape[2], k, k, stride, 0)
        for n in range(2):
            for p in range(P):
                for q in range(Q):
                    for c in range(3):
                        tot = sum(int(bs[n, p * stride + r, q * stride + s, c]) for r in range(k) for s in range(k))
                        want_b, want_c = _nearest_by_enumeration(Fraction(tot, k * k), *fmt)
                        assert by[n, p, q, c] == want_b and y[n, p, q, c] == want_c
    with pytest.raises(ValueError):
        NC.pool_np(x, fmt, "avg", 3, 2, 1)


def test_average_pool_ties():
    """Means that are exact ties of (8, 4): 2 x 2 windows summing to 4 * 33 = 132 (33 lies between 32 and 34: even field
    is 32), to 4 * 35 (-> 36), and 49-tap windows whose mean is 0.5 (-> 0) and 1.5 (-> 2)."""
    enc = lambda v: F.encode(v, 8, 4)
    x = np.array([[[[enc(32)], [enc(34)]], [[enc(32)], [enc(34)]]]], np.uint8)
    assert NC.pool_np(x, (8, 4), "avg", 2, 1, 0)[1][0, 0, 0, 0] == 32
    x = np.array([[[[enc(34)], [enc(36)]], [[enc(34)], [enc(36)]]]], np.uint8)
    assert NC.pool_np(x, (8, 4), "avg", 2, 1, 0)[1][0, 0, 0, 0] == 36
    x = np.zeros((1, 2, 2, 1), np.uint8)
    x[0, 0, 0, 0] = enc(2)
    assert NC.pool_np(x, (8, 4), "avg", 2, 1, 0)[1][0, 0, 0, 0] == 0           # 0.5 -> 0
    x[0, 0, 1, 0] = enc(4)
    assert NC.pool_np(x, (8, 4), "avg", 2, 1, 0)[1][0, 0, 0, 0] == 2           # 1.5 -> 2
    x[0, 1, 1, 0] = enc(-12)
    assert NC.pool_np(x, (8, 4), "avg", 2, 1, 0)[1][0, 0, 0, 0] == -2          # -1.5 -> -2


def _small_resnet():
    return wl.resnet50(batch=2, hw=32, classes=16)


def test_the_int8_member_reproduces_the_int8_network_oracle():
    net = _small_resnet()
    x = net.input_float()
    q8, t8 = onet.calibrate(net, x)
    qn, tn = NN.calibrate(net, x, fmt=(8, 7))
    assert qn.frac == q8.frac and qn.w_frac == q8.w_frac
    for name in q8.w:
        assert np.array_equal(NC.decode_tensor(qn.w[name], 8, 7), q8.w[name].astype(np.int64))
        assert np.array_equal(qn.b[name], q8.b[name])
    for name, v in t8.items():
        assert np.array_equal(NC.decode_tensor(tn[name], 8, 7), v.astype(np.int64)), name
    x2 = np.roll(x, 1, 0) * 0.9
    i8 = onet.infer(net, q8, x2)
    inp = NN.infer(net, qn, x2)
    for name, v in i8.items():
        assert np.array_equal(NC.decode_tensor(inp[name], 8, 7), v.astype(np.int64)), name
    assert np.array_equal(NN.logits(net, qn, inp), onet.logits(net, q8, i8))


def test_an_8_4_run_uses_its_range_and_tracks_the_float_network():
    net = _small_resnet()
    x = net.input_float()
    qz, t = NN.calibrate(net, x, fmt=(8, 4))
    bm = F.beta_max(8, 4)
    for nd in net.nodes:
        beta = NC.decode_tensor(t[nd.dst], 8, 4)
        if nd.op in ("conv", "eltwise"):
            # the scale rule puts the calibration batch's largest magnitude into the top binade of the format, unless the
            # cap at the accumulator's own scale binds
            top = int(np.abs(beta).max())
            assert top <= bm
            f_acc = (qz.frac[nd.srcs[0]] + qz.w_frac[nd.name]) if nd.op == "conv" else max(qz.frac[s] for s in nd.srcs)
            assert top >= bm // 2 or qz.frac[nd.dst] == f_acc, (nd.name, top)
        if nd.relu:
            assert beta.min() >= 0
    # inference on the calibration batch repeats the calibration tensors
    t2 = NN.infer(net, qz, x)
    for name in t:
        assert np.array_equal(t[name], t2[name])
    # against the same network in float64: the quantized logits carry its signal (4 significant bits per tensor)
    ref = _float_forward(net, x)
    got = NN.logits(net, qz, t).astype(np.float64)
    err = np.abs(got - ref).max() / np.abs(ref).max()
    assert err < 0.35, err
    assert np.corrcoef(got.ravel(), ref.ravel())[0, 1] > 0.95


def _float_forward(net, x):
    t = {net.input_name: x.astype(np.float64)}
    for nd in net.nodes:
        if nd.op == "conv":
            wf, bf = net.weights(nd)
            a = t[nd.srcs[0]]
            N, H, W, C = a.shape
            K, R, S, Cg = wf.shape
            P, Q = NC.out_hw(H, W, R, S, nd.stride, nd.pad)
            ap = np.zeros((N, H + 2 * nd.pad, W + 2 * nd.pad, C))
            ap[:, nd.pad:nd.pad + H, nd.pad:nd.pad + W] = a
            out = np.zeros((N, P, Q, K)) + bf.astype(np.float64)
            assert nd.groups == 1
            for r in range(R):
                for s in range(S):
                    out += ap[:, r:r + nd.stride * (P - 1) + 1:nd.stride, s:s + nd.stride * (Q - 1) + 1:nd.stride] @ wf[:, r, s, :].T.astype(np.float64)
            t[nd.dst] = np.maximum(out, 0) if nd.relu else out
        elif nd.op == "eltwise":
            v = t[nd.srcs[0]] + t[nd.srcs[1]]
            t[nd.dst] = np.maximum(v, 0) if nd.relu else v
        else:
            a = t[nd.srcs[0]]
            N, H, W, C = a.shape
            P, Q = NC.out_hw(H, W, nd.R, nd.R, nd.stride, nd.pad)
            ap = np.full((N, H + 2 * nd.pad, W + 2 * nd.pad, C), -np.inf if nd.op == "maxpool" else 0.0)
            ap[:, nd.pad:nd.pad + H, nd.pad:nd.pad + W] = a
            wins = [ap[:, r:r + nd.stride * (P - 1) + 1:nd.stride, s:s + nd.stride * (Q - 1) + 1:nd.stride]
                    for r in range(nd.R) for s in range(nd.R)]
            t[nd.dst] = np.max(wins, 0) if nd.op == "maxpool" else np.mean(wins, 0)
    return t[net.output_name].reshape(x.shape[0], -1)
