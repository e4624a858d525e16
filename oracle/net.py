"""Network-level oracle: single-batch calibration and inference over a layer graph.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  Follows the quantization
procedure of Sec. 3 in the paper's order, one layer at a time:

* weights: threshold = max |w| over the layer, or - with ``per_channel=True``, the
  paper's own rule - over each output channel separately; smallest power-of-two
  scale that holds it;
* bias: an integer at the product scale of input and weights;
* activations: "bootstrap" order - each layer's threshold is measured on the
  output it produces from its already-quantized upstream tensors;
* "lazy" thresholds - measured on the wide accumulator after the ReLU, only then
  is the accumulator rescaled (by a factor in (0, 1]) into the int8 output format;
* joins: element-wise add aligns both inputs exactly and rescales the sum once
  (Eq. 10); concat rescales every branch into the coarsest branch format;
  max / average pooling keep their input format.  With ``match_joins=True`` the
  scales of a concat's inputs are matched at calibration time instead (Sec. 3:
  the explicit downscale in front of a join): a convolution that feeds only the
  concat rounds its accumulators straight to the concat's format, once.

End-to-end results have no pin outside this file ("parity unpinned"); each
ingredient it calls is pinned separately.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

import oracle as orc


@dataclass
class Quantized:
    """What calibration fixes for a network: per-tensor fractional lengths and the
    integer weights / biases of every conv node."""
    frac: Dict[str, int] = field(default_factory=dict)          # tensor name -> f
    w_frac: Dict[str, object] = field(default_factory=dict)     # conv node name -> f_w (int, or int32 [K] per output channel)
    w: Dict[str, np.ndarray] = field(default_factory=dict)      # int8 [K,R,S,Cg]
    b: Dict[str, np.ndarray] = field(default_factory=dict)      # int32 [K] at f_in + f_w


def _input_codes(net, x, qz: Quantized, calibrating: bool):
    if net.input_is_int8:
        if calibrating:
            qz.frac[net.input_name] = net.f_input_codes
        return np.ascontiguousarray(x, np.int8)
    if calibrating:
        if net.fixed_f_input is not None:
            qz.frac[net.input_name] = net.fixed_f_input
        else:
            qz.frac[net.input_name] = orc.frac_from_absmax_f32(orc.absmax_f32(x))
    return orc.quantize(x, qz.frac[net.input_name])


def _float_weights(net, nd):
    """Float weights and bias of a convolution as they are quantized: with the affine layer behind it (if
    the network has such layers) folded in first - linear neighbours are combined before quantizing."""
    wf, bf = net.weights(nd)
    if getattr(net, "scale_layers", False):
        scale, shift = net.scale_shift(nd)
        wf, bf = orc.fold_scale(wf, bf, scale, shift)
    return wf, bf


def _threshold(acc, relu, rule):
    """The activation threshold of Sec. 3 in accumulator units: the maximum magnitude after the
    ReLU ("maxabs"), or the result of the histogram search of Algorithm 1 ("search")."""
    if rule == "maxabs":
        return orc.absmax_i32(acc, relu=relu)
    counts, j, m = orc.hist_i32(acc, relu=relu)
    return orc.threshold_search(counts, j, m)[0]


def lazy_pairs(net):
    """The joins that are taken at the accumulator's scale when inference runs with lazy_joins: an element-wise add of two
    different tensors one of which is the result of a convolution without activation that nothing else reads - the
    first such source in the add's own order.  Returns {name of the add node: (convolution node, the other source)}."""
    readers = {}
    for nd in net.nodes:
        for s in nd.srcs:
            readers[s] = readers.get(s, 0) + 1
    producer = {nd.dst: nd for nd in net.nodes}
    pairs = {}
    for e in net.nodes:
        if e.op != "eltwise" or e.srcs[0] == e.srcs[1]:
            continue
        for i, s in enumerate(e.srcs):
            c = producer.get(s)
            if c is not None and c.op == "conv" and not c.relu and readers[s] == 1 and s != net.output_name:
                pairs[e.name] = (c, e.srcs[1 - i])
                break
    return pairs


def _forward(net, x, qz: Quantized, calibrating: bool, per_channel: bool = False, rule: str = "maxabs",
             match_joins: bool = False, lazy_joins: bool = False):
    t = {net.input_name: _input_codes(net, x, qz, calibrating)}
    readers = {}
    for nd in net.nodes:
        for s in nd.srcs:
            readers[s] = readers.get(s, 0) + 1
    producer = {nd.dst: nd for nd in net.nodes}
    lazy = lazy_pairs(net) if (lazy_joins and not calibrating) else {}
    lazy_convs = {c.name for c, _ in lazy.values()}
    for nd in net.nodes:
        if nd.op == "conv" and nd.name in lazy_convs:
            continue                      # its accumulator goes straight into the join below; no tensor of its own
        if nd.op == "eltwise" and nd.name in lazy:
            c, other = lazy[nd.name]
            if np.ndim(qz.w_frac[c.name]) != 0:
                raise ValueError("lazy joins need one weight format per layer")
            src = c.srcs[0]
            t[nd.dst] = orc.conv_q_add_lazy(t[src], qz.w[c.name], qz.b[c.name], t[other], qz.frac[src], qz.w_frac[c.name],
                                            qz.frac[other], qz.frac[nd.dst], c.stride, c.pad, c.groups, relu=nd.relu)
            continue
        if nd.op == "conv":
            src = nd.srcs[0]
            f_in = qz.frac[src]
            if calibrating and per_channel:
                # one threshold per output channel: channel k's weights and bias get their own scale
                wf, bf = _float_weights(net, nd)
                f_wk = np.array([orc.frac_from_absmax_f32(orc.absmax_f32(wf[k])) for k in range(wf.shape[0])], np.int32)
                qz.w_frac[nd.name] = f_wk
                qz.w[nd.name] = np.stack([orc.quantize(wf[k], int(f_wk[k])) for k in range(wf.shape[0])])
                qz.b[nd.name] = np.array([orc.quantize_i32(bf[k:k + 1], f_in + int(f_wk[k]))[0] for k in range(wf.shape[0])],
                                         np.int32)
            elif calibrating:
                wf, bf = _float_weights(net, nd)
                f_w = orc.frac_from_absmax_f32(orc.absmax_f32(wf))
                qz.w_frac[nd.name] = f_w
                qz.w[nd.name] = orc.quantize(wf, f_w)
                qz.b[nd.name] = orc.quantize_i32(bf, f_in + f_w)
            f_w = qz.w_frac[nd.name]
            w, b = qz.w[nd.name], qz.b[nd.name]
            if calibrating and nd.fixed_f_out is None and np.ndim(f_w) == 1:
                # channel k's accumulators are at f_in + f_w[k]: the output format is the finest one
                # that holds every channel's post-ReLU maximum with a rescale factor in (0, 1]
                _, acc = orc.conv_q(t[src], w, b, f_in, f_w, 0, nd.stride, nd.pad, nd.groups,
                                    nd.relu, want_y=False, want_acc=True)
                m = orc.absmax_i32_channels(acc, relu=nd.relu)
                qz.frac[nd.dst] = min(orc.frac_from_absmax_i32(int(m[k]), f_in + int(f_w[k])) for k in range(len(m)))
                del acc
                t[nd.dst], _ = orc.conv_q(t[src], w, b, f_in, f_w, qz.frac[nd.dst], nd.stride, nd.pad,
                                          nd.groups, nd.relu)
            elif calibrating and nd.fixed_f_out is None:
                # threshold on the wide accumulator after the ReLU, then the one rescale of Eq. 6
                _, acc = orc.conv_q(t[src], w, b, f_in, f_w, 0, nd.stride, nd.pad, nd.groups,
                                    nd.relu, want_y=False, want_acc=True)
                m = _threshold(acc, nd.relu, rule)
                qz.frac[nd.dst] = orc.frac_from_absmax_i32(m, f_in + f_w)
                t[nd.dst] = orc.requant_i32(acc, f_in + f_w - qz.frac[nd.dst], nd.relu)
                del acc
            else:
                if calibrating:
                    qz.frac[nd.dst] = nd.fixed_f_out
                t[nd.dst], _ = orc.conv_q(t[src], w, b, f_in, f_w, qz.frac[nd.dst], nd.stride, nd.pad,
                                          nd.groups, nd.relu)
        elif nd.op == "eltwise":
            a, b = nd.srcs
            fa, fb = qz.frac[a], qz.frac[b]
            if calibrating:
                _, acc = orc.eltwise_q(t[a], fa, t[b], fb, 0, nd.relu, want_y=False, want_acc=True)
                m = _threshold(acc, nd.relu, rule)
                qz.frac[nd.dst] = orc.frac_from_absmax_i32(m, max(fa, fb))
            t[nd.dst], _ = orc.eltwise_q(t[a], fa, t[b], fb, qz.frac[nd.dst], nd.relu)
        elif nd.op == "concat":
            fs = [qz.frac[s] for s in nd.srcs]
            if calibrating:
                qz.frac[nd.dst] = nd.fixed_f_out if nd.fixed_f_out is not None else min(fs)
                if match_joins:
                    # every convolution that works for this concat alone takes the concat's format: its
                    # accumulators are rounded once, to the joined scale (never a finer one than its own)
                    for s in nd.srcs:
                        pr = producer.get(s)
                        if pr is not None and pr.op == "conv" and readers[s] == 1 and qz.frac[s] > qz.frac[nd.dst]:
                            qz.frac[s] = qz.frac[nd.dst]
                            t[s], _ = orc.conv_q(t[pr.srcs[0]], qz.w[pr.name], qz.b[pr.name], qz.frac[pr.srcs[0]],
                                                 qz.w_frac[pr.name], qz.frac[s], pr.stride, pr.pad, pr.groups, pr.relu)
                    fs = [qz.frac[s] for s in nd.srcs]
            t[nd.dst] = orc.concat_q([t[s] for s in nd.srcs], fs, qz.frac[nd.dst])
        elif nd.op in ("maxpool", "avgpool"):
            src = nd.srcs[0]
            if calibrating:
                qz.frac[nd.dst] = qz.frac[src]
            t[nd.dst] = orc.pool_q(t[src], "max" if nd.op == "maxpool" else "avg", nd.R, nd.stride, nd.pad,
                                   qz.frac[src], qz.frac[nd.dst])
        else:
            raise ValueError(nd.op)
    return t


def calibrate(net, x_calib, per_channel: bool = False, rule: str = "maxabs", match_joins: bool = False):
    """Chooses every format from ONE batch.  Returns (Quantized, tensors of that batch).
    per_channel: one weight format per output channel (Sec. 3) instead of one per layer.
    rule: "maxabs" - activation thresholds are maxima; "search" - Algorithm 1 on a histogram of the
    accumulators (per-layer weight formats only).
    match_joins: convolutions that feed only a concat produce the concat's format directly."""
    if rule not in ("maxabs", "search") or (rule == "search" and per_channel):
        raise ValueError("rule must be 'maxabs' or 'search' (the search with per-layer weight formats)")
    qz = Quantized()
    t = _forward(net, x_calib, qz, calibrating=True, per_channel=per_channel, rule=rule, match_joins=match_joins)
    return qz, t


def infer(net, qz: Quantized, x, lazy_joins: bool = False):
    """Runs the calibrated network; returns the dict of int8 tensors.
    lazy_joins: the joins lazy_pairs() lists are taken with a single rounding (the convolution's accumulator meets the
    other operand at its own scale; the convolution's int8 tensor does not exist).  The formats are those of the
    ordinary calibration."""
    return _forward(net, x, qz, calibrating=False, lazy_joins=lazy_joins)


def logits(net, qz: Quantized, tensors) -> np.ndarray:
    out = tensors[net.output_name]
    return orc.dequantize(out, qz.frac[net.output_name]).reshape(out.shape[0], -1)
