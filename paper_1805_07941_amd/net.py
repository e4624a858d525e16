"""Runs a layer graph (``workloads.Net``) on the GPU through the dfq library: the
single-batch calibration of Sec. 3 and plain inference.

This is sequencing only: which library call comes next and which buffers it gets.  Format
choices are made by ``dfq_fmt_from_absmax_*`` from thresholds the device kernels reduce;
the only host work per layer during calibration is reading one scalar back.

Order of the procedure (Sec. 3): weights get the smallest power-of-two scale that holds
max |w| of the layer (or, with ``per_channel=True``, of each output channel - the paper's own
rule); the bias becomes an integer at the product scale of input and weights;
every layer runs on its already-quantized upstream tensors ("bootstrap"); a layer's output
format is chosen from its 32-bit accumulators after the ReLU ("lazy" thresholding) with a
rescale factor in (0, 1]; element-wise adds rescale the exact aligned sum once; concat rescales
its branches into the coarsest branch format; pooling keeps its input format.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np
import torch

import ctypes as C

from . import binding as B


@dataclass
class Quantized:
    frac: Dict[str, int] = field(default_factory=dict)       # tensor name -> fractional length
    w_frac: Dict[str, object] = field(default_factory=dict)  # conv node name -> weight fractional length (int, or numpy int32 [K])
    w_frac_dev: Dict[str, torch.Tensor] = field(default_factory=dict)   # per-channel formats: the same [K] on the device
    w: Dict[str, torch.Tensor] = field(default_factory=dict)  # int8 [K,R,S,Cg] on the device
    b: Dict[str, torch.Tensor] = field(default_factory=dict)  # int32 [K] on the device


def _read_f32(t: torch.Tensor) -> float:
    return float(t.cpu()[0])


def _threshold(acc: torch.Tensor, relu: bool, rule: str) -> int:
    """Activation threshold in accumulator units: the maximum magnitude after the ReLU, or - rule
    "search" - Algorithm 1 on the histogram of the magnitudes (device histogram, host search)."""
    m = B.absmax_i32_value(B.absmax_i32(acc, relu=relu))
    if rule == "maxabs" or m == 0:
        return m
    j = B.hist_shift(m)
    counts = B.hist_i32(acc, j, relu=relu).cpu().numpy()
    return B.threshold_search(counts, j, m)[0]


def calibrate(net, x: torch.Tensor, device="cuda:0", keep_tensors: bool = True, per_channel: bool = False,
              rule: str = "maxabs", match_joins: bool = False):
    """x: float32 NHWC images (or int8 codes when the network takes codes).  Returns
    (Quantized, dict of int8 tensors of the calibration batch).
    per_channel: one weight format per output channel instead of one per layer.
    rule: "maxabs" (thresholds are maxima) or "search" (Algorithm 1; per-layer weight formats only).
    match_joins: the scales of a concat's inputs are matched at calibration time (Sec. 3: the explicit
    downscale in front of a join) - a convolution that feeds only the concat takes the concat's format and
    rounds its accumulators once, to that scale (a Plan built with fuse=True then lets it write straight
    into the joined tensor)."""
    if rule not in ("maxabs", "search") or (rule == "search" and per_channel):
        raise ValueError("rule must be 'maxabs' or 'search' (the search with per-layer weight formats)")
    qz = Quantized()
    t: Dict[str, torch.Tensor] = {}
    if net.input_is_int8:
        qz.frac[net.input_name] = net.f_input_codes
        t[net.input_name] = x
    else:
        if net.fixed_f_input is not None:
            qz.frac[net.input_name] = net.fixed_f_input
        else:
            qz.frac[net.input_name] = B.fmt_from_absmax_f32(_read_f32(B.absmax_f32(x)))
        t[net.input_name] = B.quantize(x, qz.frac[net.input_name])
    last_use = _last_use(net)
    if match_joins:
        keep_tensors = True          # a branch convolution is run again when its concat is reached
    readers: Dict[str, int] = {}
    for nd in net.nodes:
        for s in nd.srcs:
            readers[s] = readers.get(s, 0) + 1
    producer = {nd.dst: nd for nd in net.nodes}
    for idx, nd in enumerate(net.nodes):
        if nd.op == "conv":
            src = nd.srcs[0]
            f_in = qz.frac[src]
            wf, bf = net.weights(nd)
            wf = torch.from_numpy(wf).to(device)
            bf = torch.from_numpy(bf).to(device)
            if getattr(net, "scale_layers", False):
                # the affine layer behind the convolution is folded into the float weights before they are quantized
                scale, shift = net.scale_shift(nd)
                wf, bf = B.fold_scale(wf, bf, torch.from_numpy(scale).to(device), torch.from_numpy(shift).to(device))
            if per_channel:
                # channel k's weights and bias at their own scale; its accumulators are then at f_in + f_w[k],
                # and the output format is the finest that holds every channel's maximum
                gam = B.absmax_f32_rows(wf).cpu().numpy()
                f_wk = np.array([B.fmt_from_absmax_f32(float(g)) for g in gam], np.int32)
                fw_dev = torch.from_numpy(f_wk).to(device)
                qz.w_frac[nd.name], qz.w_frac_dev[nd.name] = f_wk, fw_dev
                qz.w[nd.name] = B.quantize_rows(wf, fw_dev)
                qz.b[nd.name] = B.quantize_i32_rows(bf, fw_dev, f_in)
                w, b = qz.w[nd.name], qz.b[nd.name]
                if nd.fixed_f_out is not None:
                    qz.frac[nd.dst] = nd.fixed_f_out
                else:
                    _, acc = B.conv_q_pc(t[src], w, b, f_in, fw_dev, 0, nd.stride, nd.pad, nd.groups, nd.relu,
                                         want_y=False, want_acc=True, frac_w_range=(int(f_wk.min()), int(f_wk.max())))
                    m = B.absmax_i32_channels_value(B.absmax_i32_channels(acc, relu=nd.relu))
                    del acc
                    qz.frac[nd.dst] = B.fmt_from_absmax_i32_channels(m, f_in, f_wk)
                t[nd.dst], _ = B.conv_q_pc(t[src], w, b, f_in, fw_dev, qz.frac[nd.dst], nd.stride, nd.pad, nd.groups, nd.relu,
                                           frac_w_range=(int(f_wk.min()), int(f_wk.max())))
                if not keep_tensors:
                    for s in nd.srcs:
                        if last_use.get(s) == idx and s != net.output_name:
                            t.pop(s, None)
                continue
            f_w = B.fmt_from_absmax_f32(_read_f32(B.absmax_f32(wf)))
            qz.w_frac[nd.name] = f_w
            qz.w[nd.name] = B.quantize(wf, f_w)
            qz.b[nd.name] = B.quantize_i32(bf, f_in + f_w)
            w, b = qz.w[nd.name], qz.b[nd.name]
            if nd.fixed_f_out is not None:
                qz.frac[nd.dst] = nd.fixed_f_out
            else:
                _, acc = B.conv_q(t[src], w, b, f_in, f_w, 0, nd.stride, nd.pad, nd.groups, nd.relu,
                                  want_y=False, want_acc=True)
                m = _threshold(acc, nd.relu, rule)
                del acc
                qz.frac[nd.dst] = B.fmt_from_absmax_i32(m, f_in + f_w)
            t[nd.dst], _ = B.conv_q(t[src], w, b, f_in, f_w, qz.frac[nd.dst], nd.stride, nd.pad, nd.groups, nd.relu)
        elif nd.op == "eltwise":
            a, b2 = nd.srcs
            fa, fb = qz.frac[a], qz.frac[b2]
            _, acc = B.eltwise_q(t[a], fa, t[b2], fb, 0, nd.relu, want_y=False, want_acc=True)
            m = _threshold(acc, nd.relu, rule)
            del acc
            qz.frac[nd.dst] = B.fmt_from_absmax_i32(m, max(fa, fb))
            t[nd.dst], _ = B.eltwise_q(t[a], fa, t[b2], fb, qz.frac[nd.dst], nd.relu)
        elif nd.op == "concat":
            fs = [qz.frac[s] for s in nd.srcs]
            qz.frac[nd.dst] = nd.fixed_f_out if nd.fixed_f_out is not None else min(fs)
            if match_joins:
                for s in nd.srcs:
                    pr = producer.get(s)
                    if pr is not None and pr.op == "conv" and readers[s] == 1 and qz.frac[s] > qz.frac[nd.dst]:
                        qz.frac[s] = qz.frac[nd.dst]
                        psrc = pr.srcs[0]
                        if pr.name in qz.w_frac_dev:
                            fwk = qz.w_frac[pr.name]
                            t[s], _ = B.conv_q_pc(t[psrc], qz.w[pr.name], qz.b[pr.name], qz.frac[psrc], qz.w_frac_dev[pr.name],
                                                  qz.frac[s], pr.stride, pr.pad, pr.groups, pr.relu,
                                                  frac_w_range=(int(fwk.min()), int(fwk.max())))
                        else:
                            t[s], _ = B.conv_q(t[psrc], qz.w[pr.name], qz.b[pr.name], qz.frac[psrc], qz.w_frac[pr.name],
                                               qz.frac[s], pr.stride, pr.pad, pr.groups, pr.relu)
                fs = [qz.frac[s] for s in nd.srcs]
            t[nd.dst] = B.concat_q([t[s] for s in nd.srcs], fs, qz.frac[nd.dst])
        elif nd.op in ("maxpool", "avgpool"):
            src = nd.srcs[0]
            qz.frac[nd.dst] = qz.frac[src]
            t[nd.dst] = B.pool_q(t[src], "max" if nd.op == "maxpool" else "avg", nd.R, nd.stride, nd.pad,
                                 qz.frac[src], qz.frac[nd.dst])
        else:
            raise ValueError(nd.op)
        if not keep_tensors:
            for s in nd.srcs:
                if last_use.get(s) == idx and s != net.output_name:
                    t.pop(s, None)
    return qz, t


def _last_use(net) -> Dict[str, int]:
    last = {}
    for idx, nd in enumerate(net.nodes):
        for s in nd.srcs:
            last[s] = idx
    return last


class Plan:
    """A calibrated network bound to preallocated device buffers for one batch size, so that
    a pass is a fixed sequence of library calls with no allocation and no host
    synchronization."""

    def __init__(self, net, qz: Quantized, batch: int, device="cuda:0", keep_all: bool = True, fuse: bool = False,
                 lazy_joins: bool = False):
        """fuse: the joins are merged into the convolutions in front of them (Sec. 3) where that gives the
        same bytes.  A convolution whose only consumer is the element-wise add that follows it directly
        is run together with that add by one dfq_conv_q_add call where a fused kernel covers it (the
        convolution's own int8 tensor is then never produced).  A convolution that feeds only a concat
        and already produces the concat's format writes straight into its channel slice of the joined
        tensor (no rescale is due, so no copy either); only the other branches pass through
        dfq_concat_q_into.  A convolution whose only reader is a 3x3 / 2 / pad 1 max-pooling of the same format runs
        together with it by one dfq_conv_q_maxpool call where a fused kernel covers it.
        lazy_joins (with fuse): every add of two different tensors one of which is the result of a convolution without
        activation that nothing else reads - the first such source in the add's own order - is taken with a single
        rounding by dfq_conv_q_add_lazy (a different arithmetic: the convolution's accumulator meets the other operand
        at its own scale).  Raises if the library has no kernel for one of them: there is no silent mixture."""
        self.net, self.qz, self.batch, self.device = net, qz, batch, device
        self.order = list(range(len(net.nodes)))                             # node indices in execution order
        if lazy_joins and not fuse:
            raise ValueError("lazy_joins needs fuse=True")
        self.lazy = bool(lazy_joins)
        self.fuse_input = bool(fuse)             # the input's conversion may run inside the first layer's kernel
        # conv node index -> add node index
        self.fused: Dict[int, int] = (self._lazy_pairs() if lazy_joins else self._fusable_pairs()) if fuse else {}
        if fuse:
            self.fused.update(self._pool_pairs())                            # conv node index -> max-pool node index
        self.slice_of: Dict[str, tuple] = self._direct_concat_branches() if fuse else {}   # tensor -> (joined tensor, channel offset)
        self.buf: Dict[str, torch.Tensor] = {}
        H, W, Cc = net.shapes[net.input_name]
        self.buf[net.input_name] = torch.empty((batch, H, W, Cc), dtype=torch.int8, device=device)
        if keep_all:
            for nd in net.nodes:
                if nd.dst not in self.slice_of:
                    P, Q, K = net.shapes[nd.dst]
                    self.buf[nd.dst] = torch.empty((batch, P, Q, K), dtype=torch.int8, device=device)
            for name, (dst, off) in self.slice_of.items():
                self.buf[name] = self.buf[dst][..., off:off + net.shapes[name][2]]
        else:
            self._assign_pooled()
        P, Q, K = net.shapes[net.output_name]
        self.logits = torch.empty((batch, P * Q * K), dtype=torch.float32, device=device)
        self._calls, self._calls_key, self._graph, self._keep = None, None, None, None
        self._fused_ran = None                   # after the call list is built: results of convolutions that ran fused
        self._input_in_kernel = False            # the input's conversion ran inside the first layer's kernel

    @staticmethod
    def _plain_pointwise(nd) -> bool:
        """A 1x1 convolution at stride 1 without padding or groups: the kind of layer the library's fused
        convolution + add calls exist for."""
        return nd.op == "conv" and nd.R == 1 and nd.stride == 1 and nd.pad == 0 and nd.groups == 1

    def _fusable_pairs(self) -> Dict[int, int]:
        """Convolution nodes directly followed by an element-wise add that is the only reader of
        their result (whether the library has a fused kernel for the call is probed when the call list
        is built).  Where an add is fed by two convolutions listed as (c, p, add), only c is a plain
        pointwise layer and p does not depend on c, the two are run as (p, c + add): self.order is
        changed accordingly."""
        net, qz = self.net, self.qz
        readers: Dict[str, int] = {}
        for nd in net.nodes:
            for s in nd.srcs:
                readers[s] = readers.get(s, 0) + 1
        pairs = {}
        for j in range(1, len(net.nodes)):
            e = net.nodes[j]
            if e.op != "eltwise" or e.srcs[0] == e.srcs[1]:
                continue
            c = net.nodes[j - 1]
            ok = c.op == "conv" and c.dst in e.srcs and readers.get(c.dst, 0) == 1 and c.dst != net.output_name
            if j >= 2 and ok and not self._plain_pointwise(c):
                # the convolution in front of the add is not one a fused call takes: maybe the one before it is
                c2 = net.nodes[j - 2]
                if (c2.op == "conv" and {c.dst, c2.dst} == set(e.srcs) and readers.get(c2.dst, 0) == 1
                        and c2.dst not in c.srcs and c2.dst != net.output_name and self._plain_pointwise(c2)):
                    at = self.order.index(j - 2)
                    self.order[at], self.order[at + 1] = j - 1, j - 2
                    pairs[j - 2] = j
                    continue
            if ok:
                pairs[j - 1] = j
        return pairs

    def _pool_pairs(self) -> Dict[int, int]:
        """Convolution nodes directly followed by a 3x3 / 2 / pad 1 max-pooling that is the only reader of their
        result and keeps its format: candidates for dfq_conv_q_maxpool / dfq_conv_q_pc_maxpool."""
        net, qz = self.net, self.qz
        readers: Dict[str, int] = {}
        for nd in net.nodes:
            for s in nd.srcs:
                readers[s] = readers.get(s, 0) + 1
        pairs = {}
        for j in range(1, len(net.nodes)):
            e, c = net.nodes[j], net.nodes[j - 1]
            if (e.op == "maxpool" and (e.R, e.stride, e.pad) == (3, 2, 1) and c.op == "conv" and e.srcs[0] == c.dst
                    and readers.get(c.dst, 0) == 1 and c.dst != net.output_name and c.groups == 1
                    and qz.frac[c.dst] == qz.frac[e.dst]):
                pairs[j - 1] = j
        return pairs

    def _lazy_pairs(self) -> Dict[int, int]:
        """The pairs of the single-rounding mode (see __init__); a pair whose convolution sits two nodes ahead of the add
        is run behind the node between them, which must not depend on it."""
        net, qz = self.net, self.qz
        readers: Dict[str, int] = {}
        for nd in net.nodes:
            for s in nd.srcs:
                readers[s] = readers.get(s, 0) + 1
        where = {nd.dst: i for i, nd in enumerate(net.nodes)}
        pairs = {}
        for j, e in enumerate(net.nodes):
            if e.op != "eltwise" or e.srcs[0] == e.srcs[1]:
                continue
            for s in e.srcs:
                i = where.get(s)
                c = net.nodes[i] if i is not None else None
                if c is None or c.op != "conv" or c.relu or readers[s] != 1 or s == net.output_name:
                    continue
                if c.name in qz.w_frac_dev or not self._plain_pointwise(c):
                    raise NotImplementedError("lazy join behind %s: no single-rounding kernel for this convolution" % c.name)
                if i == j - 2 and c.dst not in net.nodes[j - 1].srcs:
                    at = self.order.index(j - 2)
                    self.order[at], self.order[at + 1] = j - 1, j - 2
                elif i != j - 1:
                    raise NotImplementedError("lazy join behind %s: the convolution is not next to its add" % c.name)
                pairs[i] = j
                break
        return pairs

    def _direct_concat_branches(self) -> Dict[str, tuple]:
        """Concat inputs that a convolution produces for the concat alone, in the concat's own format."""
        net, qz = self.net, self.qz
        readers: Dict[str, int] = {}
        for nd in net.nodes:
            for s in nd.srcs:
                readers[s] = readers.get(s, 0) + 1
        producer = {nd.dst: nd for nd in net.nodes}
        out = {}
        for nd in net.nodes:
            if nd.op != "concat" or len(set(nd.srcs)) != len(nd.srcs):
                continue
            off = 0
            for s in nd.srcs:
                pr = producer.get(s)
                if (pr is not None and pr.op == "conv" and readers.get(s, 0) == 1 and s != net.output_name
                        and qz.frac[s] == qz.frac[nd.dst]):
                    out[s] = (nd.dst, off)
                off += net.shapes[s][2]
        return out

    def _assign_pooled(self):
        """Reuses buffers whose tensor is dead (sized in bytes), to keep the footprint small."""
        net = self.net
        last: Dict[str, int] = {}                # tensor name -> node index of its last reader in execution order
        for idx in self.order:
            for s in net.nodes[idx].srcs:
                last[s] = idx
        free: list = []
        owner: Dict[str, torch.Tensor] = {}
        skip = set(self.fused.values())          # an add fused into its convolution: buffer taken at the convolution
        for idx in self.order:
            nd = net.nodes[idx]
            if idx in skip:
                for s in nd.srcs:
                    if last.get(s) == idx and s in owner and s != net.input_name and s != net.output_name:
                        free.append(owner[s])
                continue
            if idx in self.fused:
                nd_dst = net.nodes[self.fused[idx]].dst
            else:
                nd_dst = nd.dst
            view_of = None
            if nd_dst in self.slice_of:
                # a branch written straight into the joined tensor: that tensor's buffer is taken now
                view_of = nd_dst
                nd_dst = self.slice_of[view_of][0]
            if nd_dst in owner:
                # (the joined tensor of a concat whose buffer an earlier branch already took)
                if view_of is not None:
                    off = self.slice_of[view_of][1]
                    self.buf[view_of] = self.buf[nd_dst][..., off:off + net.shapes[view_of][2]]
                for s in nd.srcs:
                    if last.get(s) == idx and s in owner and s != net.input_name and s != net.output_name:
                        free.append(owner[s])
                continue
            P, Q, K = net.shapes[nd_dst]
            need = self.batch * P * Q * K
            pick = None
            for i, st in enumerate(free):
                if st.numel() >= need and (pick is None or st.numel() < free[pick].numel()):
                    pick = i
            storage = free.pop(pick) if pick is not None else torch.empty(need, dtype=torch.int8, device=self.device)
            self.buf[nd_dst] = storage[:need].view(self.batch, P, Q, K)
            owner[nd_dst] = storage
            if view_of is not None:
                off = self.slice_of[view_of][1]
                self.buf[view_of] = self.buf[nd_dst][..., off:off + net.shapes[view_of][2]]
            for s in nd.srcs:
                if last.get(s) == idx and s in owner and s != net.input_name and s != net.output_name:
                    free.append(owner[s])

    def resident(self):
        """Names of the tensors whose buffer still holds them after a pass (with pooled buffers a dead
        tensor's storage is handed to a later one; a fused convolution's own result is never stored)."""
        skip = set({self.net.nodes[i].dst for i in self.fused} if self._fused_ran is None else self._fused_ran)
        if self._input_in_kernel:
            skip.add(self.net.input_name)        # converted inside the first layer's kernel, never stored
        last_at: Dict[int, str] = {}
        for name, tns in self.buf.items():          # insertion order = execution order
            if name not in skip and name not in self.slice_of:
                last_at[tns.data_ptr()] = name
        own = [n for n in self.buf if n not in skip and n not in self.slice_of and last_at[self.buf[n].data_ptr()] == n]
        return own + [n for n, (dst, _) in self.slice_of.items() if dst in own]

    # ---- execution -------------------------------------------------------------------- #
    def _build_calls(self, x: torch.Tensor):
        """The pass as a list of (C function, argument tuple) with every argument already
        marshalled except the stream, which is appended at call time."""
        L = B.lib()
        net, qz, t = self.net, self.qz, self.buf
        calls = []
        names = []         # per call: the node it belongs to (None for the input and output conversions)
        keep = []          # ctypes arrays referenced by pointer must outlive the calls
        f = B.fmt
        if net.input_is_int8:
            t[net.input_name] = x
        else:
            calls.append((L.dfq_quantize, (x.data_ptr(), t[net.input_name].data_ptr(), x.numel(), f(qz.frac[net.input_name]))))
            names.append(None)
        fused_adds = set()
        self._input_in_kernel = False
        input_readers = sum(1 for nd in net.nodes for sname in nd.srcs if sname == net.input_name)

        def ldy_of(name, K):
            # bytes between pixels of a convolution's output: its own channels, or the joined tensor's
            return int(t[self.slice_of[name][0]].shape[-1]) if name in self.slice_of else K

        for idx in self.order:
            nd = net.nodes[idx]
            if idx in fused_adds:
                continue
            partner = net.nodes[self.fused[idx]] if idx in self.fused else None
            if nd.op == "conv" and partner is not None and partner.op == "maxpool":
                # one call for the convolution and the max-pooling behind it, probed like the fused add below
                src = nd.srcs[0]
                N, H, W, Cc = t[src].shape
                K = nd.K
                pc = nd.name in qz.w_frac_dev                      # one weight format per output channel
                fn_codes = L.dfq_conv_q_pc_maxpool if pc else L.dfq_conv_q_maxpool
                fn, src_ptr = fn_codes, t[src].data_ptr()
                from_float = (src == net.input_name and not net.input_is_int8 and input_readers == 1 and calls
                              and calls[-1][0] is L.dfq_quantize)
                if from_float:
                    # the input's conversion goes into the same kernel: the float images are read directly
                    fn, src_ptr = (L.dfq_quantize_conv_q_pc_maxpool if pc else L.dfq_quantize_conv_q_maxpool), x.data_ptr()
                wfmt = ((qz.w_frac_dev[nd.name].data_ptr(), int(qz.w_frac[nd.name].min()), int(qz.w_frac[nd.name].max())) if pc
                        else (f(qz.w_frac[nd.name]),))
                args = (src_ptr, qz.w[nd.name].data_ptr(), qz.b[nd.name].data_ptr(), t[partner.dst].data_ptr(), N, H, W, Cc,
                        K, nd.R, nd.R, nd.stride, nd.pad, nd.groups, K, f(qz.frac[src])) + wfmt + (f(qz.frac[nd.dst]),
                        int(nd.relu), partner.R, partner.stride, partner.pad)
                rc = fn(*args, B._stream(None))
                if rc == B.EUNSUPPORTED and from_float:
                    fn, args = fn_codes, (t[src].data_ptr(),) + args[1:]
                    from_float = False
                    rc = fn(*args, B._stream(None))
                if rc == B.OK:
                    if from_float:
                        calls.pop()              # the separate conversion of the input
                        names.pop()
                        self._input_in_kernel = True
                    calls.append((fn, args))
                    names.append(nd.name)
                    fused_adds.add(self.fused[idx])
                    continue
                if rc != B.EUNSUPPORTED:
                    raise B.DfqError(rc, "dfq_conv_q_maxpool")
                if nd.dst not in t:
                    P, Q, Kd = net.shapes[nd.dst]
                    t[nd.dst] = torch.empty((self.batch, P, Q, Kd), dtype=torch.int8, device=self.device)
            elif nd.op == "conv" and partner is not None:
                # one call for the convolution and the add behind it; probed once here, outside any
                # capture: where no fused kernel covers the call, the two calls are issued instead
                add = partner
                other = add.srcs[0] if add.srcs[1] == nd.dst else add.srcs[1]
                src = nd.srcs[0]
                N, H, W, Cc = t[src].shape
                K = nd.K
                head = (t[src].data_ptr(), qz.w[nd.name].data_ptr(), qz.b[nd.name].data_ptr(), t[other].data_ptr(),
                        t[add.dst].data_ptr(), N, H, W, Cc, K, nd.R, nd.R, nd.stride, nd.pad, nd.groups, K, K, f(qz.frac[src]))
                tail = (f(qz.frac[nd.dst]), int(nd.relu), f(qz.frac[other]), f(qz.frac[add.dst]), int(add.relu))
                if self.lazy:
                    fn = L.dfq_conv_q_add_lazy
                    args = head + (f(qz.w_frac[nd.name]), f(qz.frac[other]), f(qz.frac[add.dst]), int(add.relu))
                    rc = fn(*args, B._stream(None))
                    if rc != B.OK:
                        raise B.DfqError(rc, "dfq_conv_q_add_lazy (%s)" % nd.name)
                    calls.append((fn, args))
                    names.append(nd.name)
                    fused_adds.add(self.fused[idx])
                    continue
                if nd.name in qz.w_frac_dev:
                    fn = L.dfq_conv_q_pc_add
                    args = head + (qz.w_frac_dev[nd.name].data_ptr(), int(qz.w_frac[nd.name].min()),
                                   int(qz.w_frac[nd.name].max())) + tail
                else:
                    fn = L.dfq_conv_q_add
                    args = head + (f(qz.w_frac[nd.name]),) + tail
                rc = fn(*args, B._stream(None))
                if rc == B.OK:
                    calls.append((fn, args))
                    names.append(nd.name)
                    fused_adds.add(self.fused[idx])
                    continue
                if rc != B.EUNSUPPORTED:
                    raise B.DfqError(rc, "dfq_conv_q_add")
                if nd.dst not in t:
                    P, Q, Kd = net.shapes[nd.dst]
                    t[nd.dst] = torch.empty((self.batch, P, Q, Kd), dtype=torch.int8, device=self.device)
            if nd.op == "conv" and nd.name in qz.w_frac_dev:
                src = nd.srcs[0]
                N, H, W, Cc = t[src].shape
                K = nd.K
                calls.append((L.dfq_conv_q_pc, (t[src].data_ptr(), qz.w[nd.name].data_ptr(), qz.b[nd.name].data_ptr(),
                                                t[nd.dst].data_ptr(), None, N, H, W, Cc, K, nd.R, nd.R, nd.stride, nd.pad,
                                                nd.groups, ldy_of(nd.dst, K), f(qz.frac[src]), qz.w_frac_dev[nd.name].data_ptr(),
                                                int(qz.w_frac[nd.name].min()), int(qz.w_frac[nd.name].max()),
                                                f(qz.frac[nd.dst]), int(nd.relu))))
            elif nd.op == "conv":
                src = nd.srcs[0]
                N, H, W, Cc = t[src].shape
                K = nd.K
                if (self.fuse_input and src == net.input_name and not net.input_is_int8 and input_readers == 1 and calls
                        and calls[-1][0] is L.dfq_quantize and nd.dst not in self.slice_of):
                    # the input's conversion inside the first layer's kernel, where the library has one for the call
                    args = (x.data_ptr(), qz.w[nd.name].data_ptr(), qz.b[nd.name].data_ptr(), t[nd.dst].data_ptr(), N, H, W, Cc, K,
                            nd.R, nd.R, nd.stride, nd.pad, nd.groups, K, f(qz.frac[src]), f(qz.w_frac[nd.name]), f(qz.frac[nd.dst]),
                            int(nd.relu))
                    rc = L.dfq_quantize_conv_q(*args, B._stream(None))
                    if rc == B.OK:
                        calls.pop()
                        names.pop()
                        self._input_in_kernel = True
                        calls.append((L.dfq_quantize_conv_q, args))
                        names.append(nd.name)
                        continue
                    if rc != B.EUNSUPPORTED:
                        raise B.DfqError(rc, "dfq_quantize_conv_q")
                calls.append((L.dfq_conv_q, (t[src].data_ptr(), qz.w[nd.name].data_ptr(), qz.b[nd.name].data_ptr(),
                                             t[nd.dst].data_ptr(), None, N, H, W, Cc, K, nd.R, nd.R, nd.stride, nd.pad,
                                             nd.groups, ldy_of(nd.dst, K), f(qz.frac[src]), f(qz.w_frac[nd.name]), f(qz.frac[nd.dst]),
                                             int(nd.relu))))
            elif nd.op == "eltwise":
                a, b2 = nd.srcs
                calls.append((L.dfq_eltwise_q, (t[a].data_ptr(), f(qz.frac[a]), t[b2].data_ptr(), f(qz.frac[b2]),
                                                t[nd.dst].data_ptr(), f(qz.frac[nd.dst]), None, t[a].numel(), int(nd.relu))))
            elif nd.op == "concat":
                # runs of neighbouring branches that still need the rescale (or a copy); branches their
                # convolution wrote straight into the joined tensor are already in place
                Ct = int(t[nd.dst].shape[-1])
                pixels = t[nd.dst].numel() // Ct
                runs, off = [], 0
                for s in nd.srcs:
                    if s not in self.slice_of:
                        if runs and runs[-1][1] == off:
                            runs[-1][2].append(s)
                            runs[-1][1] = off + int(t[s].shape[-1])
                        else:
                            runs.append([off, off + int(t[s].shape[-1]), [s]])
                    off += int(t[s].shape[-1])
                for start, _, members in runs:
                    nb = len(members)
                    ptrs = (C.c_void_p * nb)(*[t[s].data_ptr() for s in members])
                    Cs = (C.c_int * nb)(*[int(t[s].shape[-1]) for s in members])
                    fs = (B.Fmt * nb)(*[f(qz.frac[s]) for s in members])
                    keep.append((ptrs, Cs, fs))
                    calls.append((L.dfq_concat_q_into, (nb, ptrs, Cs, fs, t[nd.dst].data_ptr() + start, Ct, f(qz.frac[nd.dst]), pixels)))
                    names.append(nd.name)
                continue
            else:
                src = nd.srcs[0]
                N, H, W, Cc = t[src].shape
                mode = B.POOL_MAX if nd.op == "maxpool" else B.POOL_AVG
                calls.append((L.dfq_pool_q, (t[src].data_ptr(), t[nd.dst].data_ptr(), mode, N, H, W, Cc, nd.R, nd.stride,
                                             nd.pad, f(qz.frac[src]), f(qz.frac[nd.dst]))))
            names.append(nd.name)
        out = t[net.output_name]
        calls.append((L.dfq_dequantize, (out.data_ptr(), self.logits.data_ptr(), out.numel(), f(qz.frac[net.output_name]))))
        names.append(None)
        self._keep = keep
        self._fused_ran = {net.nodes[i].dst for i, j in self.fused.items() if j in fused_adds}
        self.call_nodes = names
        return calls

    def _calls_for(self, x: torch.Tensor):
        key = (x.data_ptr(), tuple(x.shape))
        if self._calls_key != key:
            self._calls = self._build_calls(x)
            self._calls_key = key
            self._graph = None
        return self._calls

    def run(self, x: torch.Tensor, stream=None) -> torch.Tensor:
        """One pass: x float32 images [batch,H,W,C] (or int8 codes).  Enqueues every library call
        on the stream and returns the float logits buffer (no synchronization)."""
        st = B._stream(stream)
        for fn, args in self._calls_for(x):
            rc = fn(*args, st)
            if rc != B.OK:
                raise B.DfqError(rc, fn.__name__)
        return self.logits

    def run_graph(self, x: torch.Tensor) -> torch.Tensor:
        """Same pass replayed from a HIP graph captured on first use (the call sequence is fixed and
        allocation-free, so it is capturable); removes the per-call launch cost."""
        self._calls_for(x)
        if self._graph is None:
            self.run(x)                      # first use outside capture (one-time kernel attribute set-up)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                self.run(x)
            self._graph = g
        self._graph.replay()
        return self.logits
