"""Runs a layer graph (``workloads.Net``) on the GPU with every tensor held as (8, p) dynamic floating-point codes
(Sec. 2.1, p >= 4): the single-batch calibration of Sec. 3 and plain inference, through the dfq library.

This is sequencing only: which library call comes next and which buffers it gets.  Tensors travel between the kernels as
two int8 digit planes (beta = 64 * hi + lo); codes exist at the two ends only (the quantized input and weights, the
network's output).  Scales are chosen by ``dfq_np_frac_from_absmax_*`` from thresholds the device kernels reduce:

* weights: the finest power-of-two scale that holds max |w| of the layer; bias: an integer at the product scale of input
  and weights;
* every layer runs on its already-quantized upstream tensors; its output scale comes from the largest magnitude of the
  exact accumulator after the ReLU (``dfq_conv_np_absmax`` / ``dfq_eltwise_np_absmax``) with a rescale factor in (0, 1],
  and only then is the accumulator converted, once;
* pooling keeps the scale of its input.

A stride-2 first layer over at most four channels runs on the matrix cores through the space-to-depth packing of
``dfq_stem_pack_x`` / ``dfq_stem_pack_w`` (the same integer sums).  Concat and grouped layers are not covered here.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import torch

from . import binding as B


@dataclass
class QuantizedNp:
    p: int
    frac: Dict[str, int] = field(default_factory=dict)                      # tensor name -> fractional length
    w_frac: Dict[str, int] = field(default_factory=dict)                    # conv node name -> weight fractional length
    w_codes: Dict[str, torch.Tensor] = field(default_factory=dict)          # uint8 [K,R,S,Cg]
    w: Dict[str, Tuple[torch.Tensor, torch.Tensor]] = field(default_factory=dict)   # digit planes as the kernels take them
    b: Dict[str, torch.Tensor] = field(default_factory=dict)                # int32 [K]


def packs(net, nd) -> bool:
    """A first layer the space-to-depth packing covers."""
    C = net.shapes[nd.srcs[0]][2]
    return nd.op == "conv" and nd.stride == 2 and nd.groups == 1 and C <= 4 and nd.R <= 8


def _conv_operands(net, nd, qz, src_planes):
    """(xh, xl, wh, wl, R, S, stride, pad) as the convolution call takes them."""
    wh, wl = qz.w[nd.name]
    if packs(net, nd):
        xh = B.stem_pack_x(src_planes[0], nd.R, nd.R, nd.pad)
        xl = B.stem_pack_x(src_planes[1], nd.R, nd.R, nd.pad)
        return xh, xl, wh, wl, 1, 0
    return src_planes[0], src_planes[1], wh, wl, nd.stride, nd.pad


def calibrate(net, x: torch.Tensor, p: int = 4, device="cuda:0"):
    """x: float32 NHWC images.  Returns (QuantizedNp, {tensor name: (hi, lo) digit planes of the calibration batch})."""
    if net.input_is_int8:
        raise ValueError("the (8, p) path starts from float inputs")
    qz = QuantizedNp(p=p)
    f_in = net.fixed_f_input if net.fixed_f_input is not None else B.np_frac_from_absmax_f32(float(B.absmax_f32(x).cpu()[0]), 8, p)
    qz.frac[net.input_name] = f_in
    t = {net.input_name: B.np_digits(B.quantize_np(x, 8, p, f_in), p)}
    for nd in net.nodes:
        if nd.op == "conv":
            src = nd.srcs[0]
            f_x = qz.frac[src]
            wf, bf = net.weights(nd)
            wf, bf = torch.from_numpy(wf).to(device), torch.from_numpy(bf).to(device)
            f_w = B.np_frac_from_absmax_f32(float(B.absmax_f32(wf).cpu()[0]), 8, p)
            qz.w_frac[nd.name] = f_w
            qz.w_codes[nd.name] = B.quantize_np(wf, 8, p, f_w)
            wh, wl = B.np_digits(qz.w_codes[nd.name], p)
            qz.b[nd.name] = B.quantize_i32(bf, f_x + f_w)
            K = wh.shape[0]
            if packs(net, nd):
                wh, wl = B.stem_pack_w(wh), B.stem_pack_w(wl)
            elif nd.dst == net.output_name and K % 16 and wh.shape[3] % 64 == 0 and nd.groups == 1:
                # the matrix-core kernel writes whole groups of 16 channels: the last layer gets all-zero filter rows up to
                # the next multiple (their outputs are zeros behind the real ones and are never read)
                Kp = (K + 15) // 16 * 16
                wh, wl = [torch.cat([v, torch.zeros((Kp - K,) + tuple(v.shape[1:]), dtype=v.dtype, device=device)]) for v in (wh, wl)]
                qz.b[nd.name] = torch.cat([qz.b[nd.name], torch.zeros(Kp - K, dtype=torch.int32, device=device)])
            qz.w[nd.name] = (wh, wl)
            xh, xl, wh, wl, stride, pad = _conv_operands(net, nd, qz, t[src])
            if nd.fixed_f_out is not None:
                qz.frac[nd.dst] = nd.fixed_f_out
            else:
                m = B.conv_np_absmax(xh, xl, wh, wl, qz.b[nd.name], stride, pad, nd.groups, nd.relu)
                qz.frac[nd.dst] = B.np_frac_from_absmax_u64(m, f_x + f_w, 8, p)
            _, yh, yl = B.conv_np(xh, xl, wh, wl, qz.b[nd.name], f_x, f_w, qz.frac[nd.dst], p, stride, pad, nd.groups, nd.relu,
                                  want_codes=False)
            t[nd.dst] = (yh, yl) if yh.shape[3] == K else (yh[..., :K].contiguous(), yl[..., :K].contiguous())
        elif nd.op == "eltwise":
            a, b = nd.srcs
            fa, fb = qz.frac[a], qz.frac[b]
            m = B.eltwise_np_absmax(*t[a], fa, *t[b], fb, nd.relu)
            qz.frac[nd.dst] = B.np_frac_from_absmax_u64(m, max(fa, fb), 8, p)
            _, yh, yl = B.eltwise_np(*t[a], fa, *t[b], fb, qz.frac[nd.dst], p, nd.relu, want_codes=False)
            t[nd.dst] = (yh, yl)
        elif nd.op in ("maxpool", "avgpool"):
            src = nd.srcs[0]
            qz.frac[nd.dst] = qz.frac[src]
            _, yh, yl = B.pool_np(*t[src], "max" if nd.op == "maxpool" else "avg", nd.R, nd.stride, nd.pad, p, want_codes=False)
            t[nd.dst] = (yh, yl)
        else:
            raise NotImplementedError("%s on (8, p) codes" % nd.op)
    return qz, t


class NpPlan:
    """A calibrated network bound to preallocated device buffers for one batch size: a pass is a fixed sequence of
    library calls with no allocation and no host synchronization (so it can be replayed from a HIP graph)."""

    def __init__(self, net, qz: QuantizedNp, batch: int, device="cuda:0", fuse: bool = True):
        """fuse: an element-wise add one of whose sources is the result of a convolution that nothing else reads runs in
        that convolution's epilogue (dfq_conv_np_add: the same two conversions, the convolution's own tensor is never
        stored) where the library's fused kernel covers the case; the call then stands at the add's place in the order."""
        self.net, self.qz, self.batch, self.device = net, qz, batch, device
        self.fused = self._fusable_pairs() if fuse else {}                      # add node name -> (conv node, other source)
        i8 = dict(dtype=torch.int8, device=device)
        H, W, Cc = net.shapes[net.input_name]
        self.codes_in = torch.empty((batch, H, W, Cc), dtype=torch.uint8, device=device)
        self.buf = {net.input_name: (torch.empty((batch, H, W, Cc), **i8), torch.empty((batch, H, W, Cc), **i8))}
        self.packed = {}
        for nd in net.nodes:
            P, Q, K = net.shapes[nd.dst]
            if nd.op == "conv" and not packs(net, nd):
                K = qz.w[nd.name][0].shape[0]                    # (the last layer's filters may be zero-padded)
            self.buf[nd.dst] = (torch.empty((batch, P, Q, K), **i8), torch.empty((batch, P, Q, K), **i8))
            if packs(net, nd):
                self.packed[nd.name] = (torch.empty((batch, P + 3, Q, 64), **i8), torch.empty((batch, P + 3, Q, 64), **i8))
        P, Q, K = net.shapes[net.output_name]
        Kp = self.buf[net.output_name][0].shape[3]
        if Kp != K and P * Q != 1:
            raise NotImplementedError("padded output channels behind a spatial output")
        self.codes_out = torch.empty((batch, P, Q, Kp), dtype=torch.uint8, device=device)
        self._logits_all = torch.empty((batch, P * Q * Kp), dtype=torch.float32, device=device)
        self.logits = self._logits_all[:, :P * Q * K] if Kp != K else self._logits_all
        self._calls, self._calls_key, self._graph = None, None, None

    def _fusable_pairs(self):
        net, qz = self.net, self.qz
        readers = {}
        for nd in net.nodes:
            for s_ in nd.srcs:
                readers[s_] = readers.get(s_, 0) + 1
        producer = {nd.dst: nd for nd in net.nodes}
        pairs = {}
        for e in net.nodes:
            if e.op != "eltwise" or e.srcs[0] == e.srcs[1]:
                continue
            for i, s_ in enumerate(e.srcs):
                c = producer.get(s_)
                if c is None or c.op != "conv" or readers[s_] != 1 or s_ == net.output_name or packs(net, c):
                    continue
                other = e.srcs[1 - i]
                # what dfq_conv_np_add states it covers: the matrix-core form, a downscale of the layer's own result by
                # 2^7 .. 2^36, a final factor of at most 1
                Cc = net.shapes[c.srcs[0]][2]
                K = qz.w[c.name][0].shape[0]
                mid_shift = qz.frac[c.srcs[0]] + qz.w_frac[c.name] - qz.frac[s_]
                F = max(qz.frac[s_], qz.frac[other])
                if (c.groups == 1 and Cc % 64 == 0 and K % 16 == 0 and c.R * c.R * Cc <= 13000 and 7 <= mid_shift <= 36
                        and 0 <= F - qz.frac[e.dst] <= 31 and F - qz.frac[s_] <= 18 and F - qz.frac[other] <= 18):
                    pairs[e.name] = (c, other)
                    break
        return pairs

    def _build_calls(self, x: torch.Tensor):
        L = B.lib()
        net, qz, t, p = self.net, self.qz, self.buf, self.qz.p
        ptr = lambda v: v.data_ptr() if v is not None else None
        calls, names = [], []
        xin = t[net.input_name]
        calls.append((L.dfq_quantize_np, (x.data_ptr(), ptr(self.codes_in), x.numel(), 8, p, qz.frac[net.input_name])))
        calls.append((L.dfq_np_digits, (ptr(self.codes_in), x.numel(), p, ptr(xin[0]), ptr(xin[1]))))
        names += [None, None]
        fused_convs = {c.name for c, _ in self.fused.values()}
        for nd in net.nodes:
            yh, yl = t[nd.dst]
            codes = self.codes_out if nd.dst == net.output_name else None
            if nd.op == "conv" and nd.name in fused_convs:
                continue                                            # runs at its add's place
            if nd.op == "eltwise" and nd.name in self.fused and codes is None:
                c, other = self.fused[nd.name]
                src = c.srcs[0]
                xh, xl = t[src]
                N, H, W, Cc = xh.shape
                wh, wl = qz.w[c.name]
                oh, ol = t[other]
                calls.append((L.dfq_conv_np_add, (ptr(xh), ptr(xl), ptr(wh), ptr(wl), ptr(qz.b[c.name]), ptr(oh), ptr(ol), ptr(yh), ptr(yl),
                                                  N, H, W, Cc, wh.shape[0], c.R, c.R, c.stride, c.pad, c.groups, qz.frac[src], qz.w_frac[c.name],
                                                  qz.frac[c.dst], int(c.relu), qz.frac[other], qz.frac[nd.dst], p, int(nd.relu))))
                names.append(c.name)
                continue
            if nd.op == "conv":
                src = nd.srcs[0]
                xh, xl = t[src]
                N, H, W, Cc = xh.shape
                wh, wl = qz.w[nd.name]
                R, S, stride, pad = nd.R, nd.R, nd.stride, nd.pad
                if nd.name in self.packed:
                    ph, pl = self.packed[nd.name]
                    for a, b_ in ((xh, ph), (xl, pl)):
                        calls.append((L.dfq_stem_pack_x, (ptr(a), ptr(b_), N, H, W, Cc, R, S, pad)))
                        names.append(nd.name)
                    xh, xl = ph, pl
                    N, H, W, Cc = xh.shape
                    R, S, stride, pad = 4, 1, 1, 0
                K = wh.shape[0]
                calls.append((L.dfq_conv_np, (ptr(xh), ptr(xl), ptr(wh), ptr(wl), ptr(qz.b[nd.name]), ptr(codes), ptr(yh), ptr(yl), N, H, W, Cc,
                                              K, R, S, stride, pad, nd.groups, qz.frac[src], qz.w_frac[nd.name], qz.frac[nd.dst], p,
                                              int(nd.relu))))
            elif nd.op == "eltwise":
                a, b = nd.srcs
                calls.append((L.dfq_eltwise_np, (ptr(t[a][0]), ptr(t[a][1]), qz.frac[a], ptr(t[b][0]), ptr(t[b][1]), qz.frac[b], ptr(codes),
                                                 ptr(yh), ptr(yl), qz.frac[nd.dst], p, yh.numel(), int(nd.relu))))
            elif nd.op in ("maxpool", "avgpool"):
                xh, xl = t[nd.srcs[0]]
                N, H, W, Cc = xh.shape
                calls.append((L.dfq_pool_np, (ptr(xh), ptr(xl), ptr(codes), ptr(yh), ptr(yl), B.POOL_MAX if nd.op == "maxpool" else B.POOL_AVG,
                                              N, H, W, Cc, nd.R, nd.stride, nd.pad, p)))
            else:
                raise NotImplementedError("%s on (8, p) codes" % nd.op)
            names.append(nd.name)
        calls.append((L.dfq_dequantize_np, (ptr(self.codes_out), ptr(self._logits_all), self.codes_out.numel(), 8, p, qz.frac[net.output_name])))
        names.append(None)
        self.call_nodes = names
        return calls

    def _calls_for(self, x: torch.Tensor):
        if tuple(x.shape) != tuple(self.codes_in.shape) or x.dtype != torch.float32 or not x.is_cuda or not x.is_contiguous():
            raise ValueError("x must be a contiguous float32 device tensor of the plan's input shape")
        key = x.data_ptr()
        if self._calls_key != key:
            self._calls, self._calls_key, self._graph = self._build_calls(x), key, None
        return self._calls

    def run(self, x: torch.Tensor, stream=None) -> torch.Tensor:
        """One pass over float32 images [batch,H,W,C]: enqueues every library call and returns the float logits buffer
        (no synchronization)."""
        st = B._stream(stream)
        for fn, args in self._calls_for(x):
            rc = fn(*args, st)
            if rc != B.OK:
                raise B.DfqError(rc, fn.__name__)
        return self.logits

    def run_graph(self, x: torch.Tensor) -> torch.Tensor:
        """The same pass replayed from a HIP graph captured on first use."""
        self._calls_for(x)
        if self._graph is None:
            self.run(x)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                self.run(x)
            self._graph = g
        self._graph.replay()
        return self.logits
