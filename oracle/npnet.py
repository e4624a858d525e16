"""Network-level oracle on (n, p) dynamic floating-point codes: single-batch calibration and inference over a layer graph.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).  The quantization procedure of Sec. 3, in the paper's order, with
every tensor - inputs, weights, activations - held as codes of ONE format (n, p) (Sec. 5 runs whole networks that way,
(8, 4) among them) at a power-of-two scale alpha = 2^-f of its own:

* weights: threshold = max |w| over the layer; gamma = alpha * beta_max (Sec. 2.1) gives the finest power-of-two scale
  that holds it (``npfmt.frac_from_absmax``);
* bias: an integer at the product scale of input and weights, added to the exact sum (Eq. 6);
* activations in "bootstrap" order, thresholds "lazy": the maximum magnitude of the exact accumulator after the ReLU,
  measured on the layer's already-quantized inputs, fixes the output scale (``frac_from_absmax_int``: the same rule on
  integers); only then is the accumulator converted - once - to the output format;
* element-wise add: Eq. 10 with a single conversion (``npconv.eltwise_np``), threshold on the exact sum;
* max / average pooling keep the format and scale of their input (``npconv.pool_np``).

Concatenation, grouped layers with per-channel formats and the histogram search are not part of this oracle.

End-to-end results have no pin outside this file ("parity unpinned") except for the members of the family that are int8
((8, 7)), where the whole procedure must reproduce the int8 network oracle tensor for tensor; each ingredient it calls is
pinned separately.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

import oracle as orc
from . import npconv as NC
from . import npfmt as F


@dataclass
class QuantizedNp:
    fmt: Tuple[int, int]
    frac: Dict[str, int] = field(default_factory=dict)       # tensor name -> f
    w_frac: Dict[str, int] = field(default_factory=dict)     # conv node name -> f_w
    w: Dict[str, np.ndarray] = field(default_factory=dict)   # codes [K,R,S,Cg]
    b: Dict[str, np.ndarray] = field(default_factory=dict)   # int32 [K] at f_in + f_w


def frac_from_absmax_int(m: int, f_acc: int, n: int, p: int) -> int:
    """The threshold gamma = m * 2^-f_acc of an integer tensor at scale 2^-f_acc: the largest f <= min(f_acc, 32) with
    gamma * 2^f <= beta_max, floored at -32 (gamma = alpha * beta_max of Sec. 2.1 solved for a power-of-two alpha, towards
    the coarser scale so that nothing is clipped; the rescale factor 2^(f - f_acc) stays in (0, 1] as on the int8 path).
    Python integers throughout."""
    m = int(m)
    assert m >= 0
    bm = F.beta_max(n, p)
    for f in range(min(int(f_acc), 32), -33, -1):
        if m <= (bm << (int(f_acc) - f)):
            return f
    return -32


def _forward(net, x, qz: QuantizedNp, calibrating: bool):
    n, p = qz.fmt
    fmt = qz.fmt
    if net.input_is_int8:
        raise ValueError("the (n, p) network oracle starts from float inputs")
    if calibrating:
        qz.frac[net.input_name] = (net.fixed_f_input if net.fixed_f_input is not None
                                   else F.frac_from_absmax(float(orc.absmax_f32(x)), n, p))
    t = {net.input_name: F.quantize(x, n, p, qz.frac[net.input_name])[0].astype(np.uint8)}
    for nd in net.nodes:
        if nd.op == "conv":
            src = nd.srcs[0]
            f_in = qz.frac[src]
            if calibrating:
                wf, bf = net.weights(nd)
                f_w = F.frac_from_absmax(float(orc.absmax_f32(wf)), n, p)
                qz.w_frac[nd.name] = f_w
                qz.w[nd.name] = F.quantize(wf, n, p, f_w)[0].astype(np.uint8)
                qz.b[nd.name] = orc.quantize_i32(bf, f_in + f_w)
            f_w, w, b = qz.w_frac[nd.name], qz.w[nd.name], qz.b[nd.name]
            if calibrating:
                if nd.fixed_f_out is not None:
                    qz.frac[nd.dst] = nd.fixed_f_out
                else:
                    acc = NC.conv_sum(NC.decode_tensor(t[src], *fmt), NC.decode_tensor(w, *fmt), nd.stride, nd.pad, nd.groups)
                    acc = acc + np.asarray(b, np.int64)[None, None, None, :]
                    m = int((np.maximum(acc, 0) if nd.relu else np.abs(acc)).max(initial=0))
                    qz.frac[nd.dst] = frac_from_absmax_int(m, f_in + f_w, n, p)
            t[nd.dst], _, _ = NC.conv_np(t[src], fmt, w, fmt, b, f_in + f_w - qz.frac[nd.dst], fmt, nd.stride, nd.pad,
                                         nd.groups, nd.relu)
        elif nd.op == "eltwise":
            a, b = nd.srcs
            fa, fb = qz.frac[a], qz.frac[b]
            if calibrating:
                _, _, s = NC.eltwise_np(t[a], fmt, fa, t[b], fmt, fb, fmt, max(fa, fb), nd.relu)
                m = int((np.maximum(s, 0) if nd.relu else np.abs(s)).max(initial=0))
                qz.frac[nd.dst] = frac_from_absmax_int(m, max(fa, fb), n, p)
            t[nd.dst], _, _ = NC.eltwise_np(t[a], fmt, fa, t[b], fmt, fb, fmt, qz.frac[nd.dst], nd.relu)
        elif nd.op in ("maxpool", "avgpool"):
            src = nd.srcs[0]
            if calibrating:
                qz.frac[nd.dst] = qz.frac[src]
            t[nd.dst], _ = NC.pool_np(t[src], fmt, "max" if nd.op == "maxpool" else "avg", nd.R, nd.stride, nd.pad)
        else:
            raise ValueError("%s is not part of the (n, p) network oracle" % nd.op)
    return t


def calibrate(net, x_calib, fmt=(8, 4)):
    """Chooses every scale from ONE batch.  Returns (QuantizedNp, code tensors of that batch)."""
    qz = QuantizedNp(fmt=tuple(fmt))
    return qz, _forward(net, x_calib, qz, calibrating=True)


def infer(net, qz: QuantizedNp, x):
    """Runs the calibrated network; returns the dict of code tensors (uint8)."""
    return _forward(net, x, qz, calibrating=False)


def logits(net, qz: QuantizedNp, tensors) -> np.ndarray:
    out = tensors[net.output_name]
    return F.dequantize(out, *qz.fmt, qz.frac[net.output_name]).reshape(out.shape[0], -1)
