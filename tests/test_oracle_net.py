"""Sanity of the network-level oracle (single-batch calibration, Sec. 3).

End-to-end logits have no external pin ("parity unpinned"); what the max-abs
rule implies can be checked: on the calibration batch nothing saturates, no
bit of range is wasted unless the rescale factor is capped at 1, and the
formats found are what an exact-rational evaluation of the thresholds gives.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle as orc
import oracle.net as onet
import workloads as wl


def _small_nets():
    return [wl.resnet50(batch=2, hw=32, classes=10), wl.mobilenet_v1(batch=2, hw=32, classes=10),
            wl.inception_block(batch=2, hw=8)]


@pytest.mark.parametrize("net", _small_nets(), ids=lambda n: n.name)
def test_calibration_uses_the_range_without_clipping(net):
    x = net.input_int8() if net.input_is_int8 else net.input_float()
    qz, t = onet.calibrate(net, x)
    for nd in net.nodes:
        y = t[nd.dst].astype(np.int32)
        assert y.min() >= -127
        if nd.fixed_f_out is not None or nd.op in ("maxpool", "avgpool", "concat"):
            continue
        acc_frac = (qz.frac[nd.srcs[0]] + qz.w_frac[nd.name]) if nd.op == "conv" else max(qz.frac[s] for s in nd.srcs)
        f = qz.frac[nd.dst]
        assert f <= acc_frac
        # independent check of the threshold -> format rule from the real-valued threshold
        if nd.op == "conv":
            _, acc = orc.conv_q(t[nd.srcs[0]], qz.w[nd.name], qz.b[nd.name], 0, 0, 0, nd.stride, nd.pad,
                                nd.groups, want_y=False, want_acc=True)
        else:
            a, b = nd.srcs
            F = max(qz.frac[a], qz.frac[b])
            acc = (t[a].astype(np.int64) << (F - qz.frac[a])) + (t[b].astype(np.int64) << (F - qz.frac[b]))
        acc = acc.astype(np.int64)
        if nd.relu:
            acc = np.maximum(acc, 0)
        gamma = Fraction(int(np.abs(acc).max())) / Fraction(2) ** acc_frac
        assert gamma * Fraction(2) ** f <= 127
        if f < acc_frac:
            assert gamma * Fraction(2) ** (f + 1) > 127
            assert np.abs(y).max() >= 64
    # inference on the calibration batch reproduces the calibration tensors
    t2 = onet.infer(net, qz, x)
    for k in t:
        assert np.array_equal(t[k], t2[k])
    lg = onet.logits(net, qz, t)
    assert lg.shape[0] == 2 and np.isfinite(lg).all()


def test_images_are_independent():
    net = wl.resnet50(batch=3, hw=32, classes=10)
    x = net.input_float()
    qz, _ = onet.calibrate(net, x[:2])
    full = onet.infer(net, qz, x)
    one = onet.infer(net, qz, x[2:3])
    assert np.array_equal(full[net.output_name][2:3], one[net.output_name])


def test_workload_shapes():
    r = wl.resnet50()
    assert sum(1 for n in r.nodes if n.op == "conv") == 54            # 53 convolutions + the FC layer
    assert sum(1 for n in r.nodes if n.op == "eltwise") == 16
    assert abs(r.macs_per_image() / 1e9 - 4.09) < 0.02
    m = wl.mobilenet_v1()
    assert sum(1 for n in m.nodes if n.op == "conv") == 28
    assert abs(m.macs_per_image() / 1e9 - 0.569) < 0.005
    i = wl.inception_block()
    assert i.shapes[i.output_name] == (28, 28, 256)
    assert abs(i.macs_per_image() * 64 / 1e9 - 8.86) < 0.05
    c0 = wl.config0()
    assert c0["x"].shape == (1, 32, 32, 16) and c0["w"].shape == (16, 3, 3, 16)
    l = wl.config1_layer(4, batch=1)
    assert l["x"].shape == (1, 7, 7, 512) and l["w_float"].shape == (2048, 1, 1, 512)


@pytest.mark.parametrize("net", [wl.resnet50(batch=2, hw=32, classes=10), wl.mobilenet_v1(batch=2, hw=32, classes=10)],
                         ids=lambda n: n.name)
def test_per_channel_calibration(net):
    """One weight format per output channel (the rule of Sec. 3): every channel's codes use their range,
    the output format is the finest that clips no channel of the calibration batch, and inference on
    the calibration batch reproduces its tensors."""
    x = net.input_float()
    qz, t = onet.calibrate(net, x, per_channel=True)
    qz1, _ = onet.calibrate(net, x)
    for nd in net.nodes:
        if nd.op != "conv":
            continue
        f_wk = qz.w_frac[nd.name]
        wf, _ = net.weights(nd)
        assert f_wk.shape == (wf.shape[0],)
        assert (f_wk >= qz1.w_frac[nd.name]).all()                 # never coarser than the per-layer format
        for k in range(wf.shape[0]):
            g = Fraction(float(np.abs(wf[k]).max()))
            if g == 0:
                continue
            assert g * Fraction(2) ** int(f_wk[k]) <= 127 < g * Fraction(2) ** (int(f_wk[k]) + 1)
        if nd.fixed_f_out is not None:
            continue
        f_in, f = qz.frac[nd.srcs[0]], qz.frac[nd.dst]
        _, acc = orc.conv_q(t[nd.srcs[0]], qz.w[nd.name], qz.b[nd.name], 0, 0, 0, nd.stride, nd.pad, nd.groups,
                            want_y=False, want_acc=True)
        acc = acc.astype(np.int64)
        if nd.relu:
            acc = np.maximum(acc, 0)
        m = np.abs(acc).reshape(-1, acc.shape[-1]).max(axis=0)
        gam = [Fraction(int(m[k])) / Fraction(2) ** (f_in + int(f_wk[k])) for k in range(len(m))]
        assert all(gk * Fraction(2) ** f <= 127 for gk in gam)
        assert f <= f_in + int(f_wk.min())
        if f < f_in + int(f_wk.min()):
            assert any(gk * Fraction(2) ** (f + 1) > 127 for gk in gam)
    t2 = onet.infer(net, qz, x)
    for k in t:
        assert np.array_equal(t[k], t2[k])


def test_threshold_search_calibration():
    """Activation thresholds from Algorithm 1 instead of the maximum: a threshold never exceeds the
    maximum, so no format gets coarser; weights and the bootstrap order are unchanged."""
    net = wl.resnet50(batch=2, hw=32, classes=10)
    x = net.input_float()
    qz0, _ = onet.calibrate(net, x)
    qz, t = onet.calibrate(net, x, rule="search")
    assert qz.w_frac[net.nodes[0].name] == qz0.w_frac[net.nodes[0].name]
    finer = 0
    for nd in net.nodes:
        if nd.op in ("conv", "eltwise") and nd.fixed_f_out is None:
            acc_frac = (qz.frac[nd.srcs[0]] + qz.w_frac[nd.name]) if nd.op == "conv" else max(qz.frac[s] for s in nd.srcs)
            assert qz.frac[nd.dst] <= acc_frac
        assert int(t[nd.dst].astype(np.int32).min()) >= -127
    # the first layers see identical inputs under both rules: there the searched format is the same or finer
    first = net.nodes[0]
    assert qz.frac[first.dst] >= qz0.frac[first.dst]
    t2 = onet.infer(net, qz, x)
    for k in t:
        assert np.array_equal(t[k], t2[k])
    with pytest.raises(ValueError):
        onet.calibrate(net, x, per_channel=True, rule="search")


def test_matched_join_scales():
    """match_joins (Sec. 3: the scales of a join's inputs are matched; explicit downscale in front of the join): every
    convolution that feeds only the concat ends at the concat's format, its slice of the joined tensor is its
    accumulator rounded ONCE to that format (Fraction check on sampled elements), the concat is then a plain copy,
    and nothing upstream of the branches changes."""
    net = wl.inception_block(batch=2, hw=8)
    x = net.input_int8()
    qz0, t0 = onet.calibrate(net, x)
    qz1, t1 = onet.calibrate(net, x, match_joins=True)
    cat = net.nodes[-1]
    f_cat = qz1.frac[cat.dst]
    assert f_cat == qz0.frac[cat.dst] == min(qz0.frac[s] for s in cat.srcs)
    assert any(qz0.frac[s] != f_cat for s in cat.srcs)                     # the default calibration does rescale some branch
    producer = {nd.dst: nd for nd in net.nodes}
    off = 0
    rng = np.random.default_rng(5)
    for s in cat.srcs:
        nd = producer[s]
        assert qz1.frac[s] == f_cat
        assert np.array_equal(t1[cat.dst][..., off:off + nd.K], t1[s])         # copy, no second rounding
        src = nd.srcs[0]
        assert np.array_equal(t1[src], t0[src]) and qz1.frac[src] == qz0.frac[src]
        _, acc = orc.conv_q(t1[src], qz1.w[nd.name], qz1.b[nd.name], 0, 0, 0, nd.stride, nd.pad, nd.groups, want_y=False,
                            want_acc=True)
        f_acc = qz1.frac[src] + qz1.w_frac[nd.name]
        flat, out = acc.reshape(-1), t1[s].reshape(-1)
        for i in rng.integers(0, flat.size, 200):
            v = Fraction(max(int(flat[i]), 0) if nd.relu else int(flat[i])) * Fraction(2) ** (f_cat - f_acc)
            lo = v.numerator // v.denominator
            r = v - lo
            want = lo + (1 if (r > Fraction(1, 2) or (r == Fraction(1, 2) and lo % 2)) else 0)
            assert int(out[i]) == max(-127, min(127, want))
        off += nd.K
    # inference reproduces the calibration tensors with the matched formats as well
    t2 = onet.infer(net, qz1, x)
    for k in t1:
        assert np.array_equal(t1[k], t2[k])


def test_scale_layers_are_folded_before_quantizing():
    """A network with an affine layer behind every convolution calibrates through the folding pre-pass: the integer
    weights are the quantized folded weights, and the folding changes them."""
    plain = wl.resnet50(batch=2, hw=32, classes=10)
    net = wl.resnet50(batch=2, hw=32, classes=10, scale_layers=True)
    x = net.input_float()
    qz, t = onet.calibrate(net, x)
    qz0, _ = onet.calibrate(plain, x)
    nd = net.nodes[0]
    wf, bf = net.weights(nd)
    scale, shift = net.scale_shift(nd)
    w2, b2 = orc.fold_scale(wf, bf, scale, shift)
    f_w = orc.frac_from_absmax_f32(orc.absmax_f32(w2))
    assert qz.w_frac[nd.name] == f_w and np.array_equal(qz.w[nd.name], orc.quantize(w2, f_w))
    assert np.array_equal(qz.b[nd.name], orc.quantize_i32(b2, qz.frac["input"] + f_w))
    assert not np.array_equal(qz.w[nd.name], qz0.w[nd.name])
    assert np.isfinite(onet.logits(net, qz, t)).all()


def test_lazy_joins_are_single_roundings_of_the_listed_pairs():
    """Inference with lazy_joins: the sixteen joins of the ResNet-50-shaped graph pair with the third convolution of their
    block (the first listed source that qualifies, also where a projection qualifies too); the paired convolutions leave
    no tensor; everything in front of the first join is untouched; the first join is the oracle's single-rounding call
    on the same operands; the results differ from ordinary inference, by little."""
    net = wl.resnet50(batch=2, hw=32, classes=10)
    x = net.input_float()
    qz, _ = onet.calibrate(net, x)
    std = onet.infer(net, qz, x)
    lazy = onet.infer(net, qz, x, lazy_joins=True)
    pairs = onet.lazy_pairs(net)
    adds = [nd for nd in net.nodes if nd.op == "eltwise"]
    assert len(adds) == 16 and set(pairs) == {e.name for e in adds}
    assert all(c.name.endswith("_c") for c, _ in pairs.values())
    assert all(c.dst not in lazy for c, _ in pairs.values()) and all(e.dst in lazy for e in adds)
    first = adds[0]
    for nd in net.nodes:
        if nd is first:
            break
        if nd.dst in lazy:
            assert np.array_equal(lazy[nd.dst], std[nd.dst]), nd.name
    c, other = pairs[first.name]
    want = orc.conv_q_add_lazy(std[c.srcs[0]], qz.w[c.name], qz.b[c.name], std[other], qz.frac[c.srcs[0]], qz.w_frac[c.name],
                               qz.frac[other], qz.frac[first.dst], c.stride, c.pad, c.groups, relu=first.relu)
    assert np.array_equal(lazy[first.dst], want)
    d = np.abs(lazy[first.dst].astype(np.int16) - std[first.dst].astype(np.int16))
    assert 0 < (d != 0).mean() < 0.5 and np.percentile(d, 99) <= 1
    # calibration does not know the mode: same formats either way
    qz2, _ = onet.calibrate(net, x)
    assert qz2.frac == qz.frac
