#!/usr/bin/env python3
"""Benchmark of the quantized-inference hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch that is already resident in
HBM: quantize the float images, run every int8 layer of the ResNet-50-shaped network
(53 convolutions + the fully connected layer, 16 residual adds, max and average pooling),
dequantize the logits.  Formats, integer weights and biases come from a single-batch
calibration done before the timed region.

Prints ONE JSON line.  `value` is int8 TOPS of the whole step (2 x multiply-accumulates of all
convolution layers / step time); images/s, the roofline of the matrix-core convolution kernel
(HIP events around each of its launches, inside the timed region) and the CPU oracle timed on a
bounded sample of the same workload are carried alongside.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8 matrix peak, published
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def conv_nodes(net):
    return [nd for nd in net.nodes if nd.op == "conv"]


def node_macs(net, nd):
    C = net.shapes[nd.srcs[0]][2]
    P, Q, K = net.shapes[nd.dst]
    return P * Q * K * nd.R * nd.R * (C // nd.groups)


def node_bytes(net, nd):
    """Algorithmic HBM bytes per image of one conv: int8 input + int8 output (weights and bias
    are added once per launch by the caller)."""
    H, W, C = net.shapes[nd.srcs[0]]
    P, Q, K = net.shapes[nd.dst]
    return H * W * C + P * Q * K


def cpu_baseline(net, batch_sample: int, calib_n: int, per_channel: bool = False, lazy_joins: bool = False):
    """The oracle as it stands, on the host cores: inference of `batch_sample` images."""
    import oracle as orc
    import oracle.net as onet
    x = net.input_float()
    qz, _ = onet.calibrate(net, x[:calib_n], per_channel=per_channel)
    xs = x[:batch_sample]
    t0 = time.perf_counter()
    t = onet.infer(net, qz, xs, lazy_joins=lazy_joins)
    ref_logits = onet.logits(net, qz, t)
    dt = time.perf_counter() - t0
    macs = net.macs_per_image() * batch_sample
    return ref_logits, dict(value=2 * macs / dt / 1e12, unit="TOPS", cores=orc.num_threads(), kind="oracle",
                sample=f"inference of {batch_sample} of the {net.batch} images (same network, same formats rule), "
                       f"{dt:.2f} s", images_per_s=batch_sample / dt)


def bench_layers(args):
    """The five dense layers of configs[1] on their own at the given batch: formats from the library's own
    single-batch calibration of each layer, four rotating sets of input / output buffers (together larger
    than the 256 MB last-level cache at batch 256), HIP events over 20 launches.  One JSON line."""
    import numpy as np
    import torch
    import workloads as wl
    from paper_1805_07941_amd import binding as B

    dev = "cuda:0"
    rows = []
    layer_set = {"3x3": wl.RESNET_3X3_SET, "grouped": wl.GROUPED_SET, "first": wl.FIRST_LAYER_SET}.get(args.layer_set, wl.RESNET_LAYER_SET)
    for i in range(len(layer_set)):
        L = wl.config1_layer(i, batch=args.batch, layer_set=layer_set)
        wf, bf = torch.from_numpy(L["w_float"]).to(dev), torch.from_numpy(L["b_float"]).to(dev)
        f_in, pad, stride, groups = L["f_in"], L["pad"], L["stride"], L["groups"]
        f_w = B.fmt_from_absmax_f32(float(B.absmax_f32(wf).cpu()[0]))
        w, b = B.quantize(wf, f_w), B.quantize_i32(bf, f_in + f_w)
        x0 = torch.from_numpy(L["x"]).to(dev)
        _, acc = B.conv_q(x0[:8].contiguous(), w, b, f_in, f_w, 0, stride, pad, groups, True, want_y=False, want_acc=True)
        f_out = B.fmt_from_absmax_i32(B.absmax_i32_value(B.absmax_i32(acc, relu=True)), f_in + f_w)
        del acc
        nset = 4
        xs = [x0] + [x0.roll(k + 1, 0).contiguous() for k in range(nset - 1)]
        N, H, W, C = x0.shape
        K, R = w.shape[0], w.shape[1]
        P, Q = B.conv_out_hw(H, W, R, R, stride, pad)
        ys = [torch.empty((N, P, Q, K), dtype=torch.int8, device=dev) for _ in range(nset)]
        for k in range(3):
            B.conv_q(xs[k % nset], w, b, f_in, f_w, f_out, stride, pad, groups, True, out=ys[k % nset])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        iters = args.steps
        e0.record()
        for k in range(iters):
            B.conv_q(xs[k % nset], w, b, f_in, f_w, f_out, stride, pad, groups, True, out=ys[k % nset])
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        ops = 2.0 * N * P * Q * K * R * R * (C // groups)
        by = x0.numel() + ys[0].numel() + w.numel() + 4 * K
        t_roof = max(ops / (INT8_MFMA_PEAK_TOPS * 1e12), by / (HBM_PEAK_GBS * 1e9)) * 1e3
        rows.append(dict(layer=L["name"], shape="%dx%dx%d -> %d, %dx%d%s" % (H, W, C, K, R, R, "" if groups == 1 else " /%d g%d" % (stride, groups)),
                         kernel=B.CONV_VARIANT_NAMES[B.conv_q_select(N, H, W, C, K, R, R, stride, pad, groups)], us=round(ms * 1e3, 1),
                         tops=round(ops / ms / 1e9, 1), gbs=round(by / ms / 1e6, 1),
                         pct_mfma_peak=round(100 * ops / ms / 1e9 / INT8_MFMA_PEAK_TOPS, 1),
                         pct_hbm_peak=round(100 * by / ms / 1e6 / HBM_PEAK_GBS, 1), pct_roofline=round(100 * t_roof / ms, 1)))
        if args.layer_set == "first":
            # the 3x3 / 2 / pad 1 max-pooling behind the layer: as a second call, and inside the convolution's kernel
            PP, PQ = B.conv_out_hw(P, Q, 3, 3, 2, 1)
            ps = [torch.empty((N, PP, PQ, K), dtype=torch.int8, device=dev) for _ in range(nset)]

            def timed(fn):
                for k in range(3):
                    fn(k)
                torch.cuda.synchronize()
                e0.record()
                for k in range(iters):
                    fn(k)
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / iters

            ms_pool = timed(lambda k: B.pool_q(ys[k % nset], "max", 3, 2, 1, f_out, f_out, out=ps[k % nset]))
            fused_ok = B.conv_q_maxpool(xs[0], w, b, f_in, f_w, f_out, stride, pad, True, out=ps[0]) is not None
            by_pool = ys[0].numel() + ps[0].numel()
            rows.append(dict(layer=L["name"] + " max-pool alone", shape="%dx%dx%d -> %dx%d, 3x3 /2" % (P, Q, K, PP, PQ), kernel="dfq_pool_q",
                             us=round(ms_pool * 1e3, 1), gbs=round(by_pool / ms_pool / 1e6, 1), pct_hbm_peak=round(100 * by_pool / ms_pool / 1e6 / HBM_PEAK_GBS, 1)))
            if fused_ok:
                ms_f = timed(lambda k: B.conv_q_maxpool(xs[k % nset], w, b, f_in, f_w, f_out, stride, pad, True, out=ps[k % nset]))
                by_f = x0.numel() + ps[0].numel() + w.numel() + 4 * K
                rows.append(dict(layer=L["name"] + " + max-pool in one kernel", shape="%dx%dx%d -> %dx%dx%d" % (H, W, C, PP, PQ, K), kernel="dfq_conv_q_maxpool",
                                 us=round(ms_f * 1e3, 1), tops=round(ops / ms_f / 1e9, 1), gbs=round(by_f / ms_f / 1e6, 1),
                                 pct_mfma_peak=round(100 * ops / ms_f / 1e9 / INT8_MFMA_PEAK_TOPS, 1),
                                 pct_hbm_peak=round(100 * by_f / ms_f / 1e6 / HBM_PEAK_GBS, 1),
                                 two_calls_us=round((ms + ms_pool) * 1e3, 1)))
                # ... and with the conversion of the float images in front taken into the kernel as well
                xf = [(t.float() * 2.0 ** -f_in).contiguous() for t in xs]           # exact: converts back to the same codes
                qs = [torch.empty_like(t) for t in xs]
                ms_q = timed(lambda k: B.quantize(xf[k % nset], f_in, out=qs[k % nset]))
                rows.append(dict(layer=L["name"] + " input conversion alone", shape="%dx%dx%d float -> int8" % (H, W, C), kernel="dfq_quantize",
                                 us=round(ms_q * 1e3, 1), gbs=round(5 * x0.numel() / ms_q / 1e6, 1),
                                 pct_hbm_peak=round(100 * 5 * x0.numel() / ms_q / 1e6 / HBM_PEAK_GBS, 1)))
                if B.conv_q_maxpool(xf[0], w, b, f_in, f_w, f_out, stride, pad, True, out=ps[0]) is not None:
                    ms_qf = timed(lambda k: B.conv_q_maxpool(xf[k % nset], w, b, f_in, f_w, f_out, stride, pad, True, out=ps[k % nset]))
                    by_qf = 4 * x0.numel() + ps[0].numel() + w.numel() + 4 * K
                    rows.append(dict(layer=L["name"] + " conversion + layer + max-pool in one kernel", shape="%dx%dx%d float -> %dx%dx%d" % (H, W, C, PP, PQ, K),
                                     kernel="dfq_quantize_conv_q_maxpool", us=round(ms_qf * 1e3, 1), tops=round(ops / ms_qf / 1e9, 1),
                                     gbs=round(by_qf / ms_qf / 1e6, 1), pct_mfma_peak=round(100 * ops / ms_qf / 1e9 / INT8_MFMA_PEAK_TOPS, 1),
                                     pct_hbm_peak=round(100 * by_qf / ms_qf / 1e6 / HBM_PEAK_GBS, 1),
                                     two_calls_us=round((ms_q + ms + ms_pool) * 1e3, 1)))
                del xf, qs
            del ps
        del xs, ys, x0
    what = {"3x3": "the four 3x3 shapes of the ResNet-50-shaped network", "grouped": "grouped and depthwise shapes",
            "first": "first layers (3 channels, stride 2) with the max-pooling behind them"}.get(args.layer_set, "configs[1]")
    print(json.dumps({"metric": "int8 conv TOPS per layer of %s, standalone, b=%d" % (what, args.batch), "unit": "TOPS",
                      "n_gpus": 1, "dtype": "int8", "data": "synthetic", "buffers": "4 rotating sets per layer", "layers": rows}))


def bench_layers_np(args):
    """The same layer shapes on (8, 4) dynamic floating-point codes (dfq_conv_np: digit planes in, digit planes out):
    activations and weights of the int8 layer set re-quantized to (8, 4) by the library's own kernels, output format from
    a first pass at a scale that cannot saturate.  One JSON line; `tops` counts the products of Eq. 6 (2 ops each), the
    matrix cores execute four int8 products for every one of them."""
    import torch
    import workloads as wl
    from paper_1805_07941_amd import binding as B

    dev = "cuda:0"
    rows = []
    layer_set = wl.RESNET_3X3_SET if args.layer_set == "3x3" else wl.RESNET_LAYER_SET
    for i in range(len(layer_set)):
        L = wl.config1_layer(i, batch=args.batch, layer_set=layer_set)
        wf, bf = torch.from_numpy(L["w_float"]).to(dev), torch.from_numpy(L["b_float"]).to(dev)
        pad = L["pad"]
        xf = B.dequantize(torch.from_numpy(L["x"]).to(dev), L["f_in"])
        f_x = B.np_frac_from_absmax_f32(float(B.absmax_f32(xf).cpu()[0]), 8, 4)
        f_w = B.np_frac_from_absmax_f32(float(B.absmax_f32(wf).cpu()[0]), 8, 4)
        xh, xl = B.np_digits(B.quantize_np(xf, 8, 4, f_x), 4)
        wh, wl_ = B.np_digits(B.quantize_np(wf, 8, 4, f_w), 4)
        b = B.quantize_i32(bf, f_x + f_w)
        del xf
        N, H, W, C = xh.shape
        K, R = wh.shape[0], wh.shape[1]
        # first pass on the calibration images at a scale no sum can saturate (|acc| <= terms * 1984^2), then the threshold
        shift0 = int(math.ceil(math.log2(R * R * C * 1984.0)))
        y0, _, _ = B.conv_np(xh[:8].contiguous(), xl[:8].contiguous(), wh, wl_, b, f_x, f_w, f_x + f_w - shift0, 4, 1, pad, 1, True,
                             want_digits=False)
        gamma = float(B.absmax_f32(B.dequantize_np(y0, 8, 4, f_x + f_w - shift0)).cpu()[0]) * (1.0 + 1.0 / 16)   # one step of slack
        f_y = min(B.np_frac_from_absmax_f32(gamma, 8, 4), f_x + f_w + 16)
        nset = 4
        xhs = [xh] + [xh.roll(k + 1, 0).contiguous() for k in range(nset - 1)]
        xls = [xl] + [xl.roll(k + 1, 0).contiguous() for k in range(nset - 1)]
        outs = [(None, torch.empty((N, H, W, K), dtype=torch.int8, device=dev), torch.empty((N, H, W, K), dtype=torch.int8, device=dev))
                for _ in range(nset)]
        run = lambda k: B.conv_np(xhs[k % nset], xls[k % nset], wh, wl_, b, f_x, f_w, f_y, 4, 1, pad, 1, True, out=outs[k % nset])
        for k in range(3):
            run(k)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        iters = args.steps
        e0.record()
        for k in range(iters):
            run(k)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        ops = 2.0 * N * H * W * K * R * R * C
        by = 2 * xh.numel() + 2 * outs[0][1].numel() + 2 * wh.numel() + 4 * K
        t_roof = max(4 * ops / (INT8_MFMA_PEAK_TOPS * 1e12), by / (HBM_PEAK_GBS * 1e9)) * 1e3
        nonzero = float((outs[0][1] != 0).logical_or(outs[0][2] != 0).float().mean().cpu())
        rows.append(dict(layer=L["name"], shape="%dx%dx%d -> %d, %dx%d" % (H, W, C, K, R, R), kernel="np-mfma", us=round(ms * 1e3, 1),
                         tops=round(ops / ms / 1e9, 1), int8_matrix_tops=round(4 * ops / ms / 1e9, 1), gbs=round(by / ms / 1e6, 1),
                         pct_mfma_peak=round(100 * 4 * ops / ms / 1e9 / INT8_MFMA_PEAK_TOPS, 1),
                         pct_hbm_peak=round(100 * by / ms / 1e6 / HBM_PEAK_GBS, 1), pct_roofline=round(100 * t_roof / ms, 1),
                         formats=dict(f_x=f_x, f_w=f_w, f_y=f_y), nonzero_outputs=round(nonzero, 3)))
        del xhs, xls, outs, xh, xl
    # the residual joins of the same network on (8, 4) codes (dfq_eltwise_np: four planes in, two out, 6 B per element)
    joins = []
    gen = torch.Generator(device=dev).manual_seed(1)
    for H, C in ((56, 256), (28, 512), (14, 1024), (7, 2048)):
        shape = (args.batch, H, H, C)
        codes = [torch.randint(0, 256, shape, dtype=torch.uint8, device=dev, generator=gen) for _ in range(2)]
        (ah, al), (bh, bl) = [B.np_digits(c, 4) for c in codes]
        del codes
        yh, yl = torch.empty_like(ah), torch.empty_like(ah)
        L = B.lib()
        st = torch.cuda.current_stream().cuda_stream
        run = lambda: L.dfq_eltwise_np(ah.data_ptr(), al.data_ptr(), 9, bh.data_ptr(), bl.data_ptr(), 8, None, yh.data_ptr(), yl.data_ptr(), 8, 4,
                                       ah.numel(), 1, st)
        for _ in range(3):
            assert run() == B.OK
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        by = 6 * ah.numel()
        joins.append(dict(shape="%dx%dx%d" % (H, H, C), us=round(ms * 1e3, 1), gbs=round(by / ms / 1e6, 1),
                          pct_hbm_peak=round(100 * by / ms / 1e6 / HBM_PEAK_GBS, 1)))
        del ah, al, bh, bl, yh, yl
    what = "the four 3x3 shapes of the ResNet-50-shaped network" if args.layer_set == "3x3" else "configs[1]"
    print(json.dumps({"joins": joins, "metric": "(8,4) dynamic floating-point conv TOPS per dense layer of %s, standalone, b=%d" % (what, args.batch),
                      "unit": "TOPS", "n_gpus": 1, "dtype": "(8,4) codes as two int8 digit planes, three int32 accumulators -> exact 64-bit sum",
                      "data": "synthetic", "buffers": "4 rotating sets per layer",
                      "roofline_note": "pct_mfma_peak prices the four int8 matrix products per block against 5 POP/s", "layers": rows}))


def bench_net_np(args):
    """The ResNet-50-shaped pass with every tensor on (8, 4) dynamic floating-point codes (npnet.NpPlan): single-batch
    calibration on --calib images, the pass replayed from a HIP graph, then - outside the timed region - the duration of
    every library call of one pass (event pairs on the launch stream) and the logits of a few images against the
    network oracle on (8, 4) codes, which calibrates for itself.  One JSON line."""
    import numpy as np
    import torch
    import workloads as wl
    from paper_1805_07941_amd import binding as B
    from paper_1805_07941_amd import npnet

    dev = "cuda:0"
    net = wl.resnet50(batch=args.batch)
    x_host = net.input_float()
    x = torch.from_numpy(x_host).to(dev)
    qz, _ = npnet.calibrate(net, x[:args.calib].contiguous(), p=4)
    plan = npnet.NpPlan(net, qz, args.batch)
    step = (lambda: plan.run(x)) if args.no_graph else (lambda: plan.run_graph(x))
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3

    calls = plan._calls_for(x)
    st = B._stream(None)
    reps = max(2, min(args.steps, 5))
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in calls] for _ in range(reps)]
    for r in range(reps):
        torch.cuda._sleep(6_000_000)
        for (fn, cargs), (e0, e1) in zip(calls, evs[r]):
            e0.record()
            rc = fn(*cargs, st)
            e1.record()
            if rc != B.OK:
                raise B.DfqError(rc, fn.__name__)
    torch.cuda.synchronize()
    node = {nd.name: nd for nd in net.nodes}
    by_fn, layers = {}, []
    for i, ((fn, _), name) in enumerate(zip(calls, plan.call_nodes)):
        us = sum(evs[r][i][0].elapsed_time(evs[r][i][1]) for r in range(reps)) / reps * 1e3
        d = by_fn.setdefault(fn.__name__, dict(calls=0, us=0.0))
        d["calls"] += 1
        d["us"] = round(d["us"] + us, 1)
        if fn.__name__ in ("dfq_conv_np", "dfq_conv_np_add"):
            nd = node[name]
            o = 2.0 * node_macs(net, nd) * args.batch
            layers.append(dict(layer=name, us=round(us, 1), tops=round(o / us / 1e6, 1), int8_matrix_tops=round(4 * o / us / 1e6, 1)))
    macs_step = net.macs_per_image() * args.batch
    tops = 2 * macs_step / (ms_per_step * 1e-3) / 1e12
    conv_us = by_fn["dfq_conv_np"]["us"] + by_fn.get("dfq_conv_np_add", dict(us=0.0))["us"]
    n_conv = by_fn["dfq_conv_np"]["calls"] + by_fn.get("dfq_conv_np_add", dict(calls=0))["calls"]

    cpu, parity_checked = None, None
    if args.cpu_sample > 0:
        import oracle.npnet as NN
        n_cpu = min(args.cpu_sample, 4, args.batch)
        n_cal = min(args.calib, args.batch)
        oq, _ = NN.calibrate(net, x_host[:n_cal], fmt=(8, 4))
        t1 = time.perf_counter()
        ref = NN.logits(net, oq, NN.infer(net, oq, x_host[:n_cpu]))
        t_cpu = time.perf_counter() - t1
        got = step().cpu().numpy()[:n_cpu]
        equal = int(sum(bool(np.array_equal(got[i], ref[i])) for i in range(n_cpu)))
        parity_checked = dict(images=n_cpu, images_with_identical_logits=equal, tolerance=0,
                              what="float logits of the timed plan against the (8, 4) network oracle's")
        cpu = dict(value=round(n_cpu / t_cpu, 3), unit="images/s", cores=os.cpu_count(), kind="oracle",
                   sample="%d images of the same batch through oracle.npnet.infer (numpy; window sums by the double matrix product)" % n_cpu)
    line = {
        "metric": "(8,4) dynamic floating-point conv TOPS (2*MAC/s of Eq. 6's products), whole ResNet-50-shaped pass, b=%d" % args.batch,
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "(8,4) codes as two int8 digit planes; four int8 matrix products per block into three int32 accumulators -> exact sum",
        "data": "synthetic", "launch": "per-call from Python" if args.no_graph else "HIP graph replay of the fixed call sequence",
        "config": {"workload": "configs[4]'s network on (8, 4) codes: ResNet-50-shaped, 224x224x3, batch %d, scales from a single-batch "
                               "calibration on %d images" % (args.batch, args.calib), "global_batch": args.batch},
        "images_per_s": round(args.batch / (ms_per_step * 1e-3), 1),
        "roofline": {"bound": "mfma", "kernel": "conv_np_mfma_kernel: the %d convolution launches of a pass (%d of them with the residual add in the epilogue)" % (n_conv, len(plan.fused)),
                     "achieved": round(4 * 2 * macs_step / conv_us / 1e6, 1), "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(4 * 2 * macs_step / conv_us / 1e6 / INT8_MFMA_PEAK_TOPS, 4),
                     "note": "int8 matrix operations executed (four per product of Eq. 6) over the summed event intervals of the convolution calls",
                     "traffic": None},
        "calls": by_fn, "cpu_baseline": cpu, "parity_checked": parity_checked, "conv_layers": layers,
    }
    return line


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--calib", type=int, default=8, help="images of the single calibration batch")
    ap.add_argument("--cpu-sample", type=int, default=128, help="images the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--no-kernel-events", action="store_true", help="skip the per-launch events (pure step timing)")
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of replaying a HIP graph")
    ap.add_argument("--no-fuse", action="store_true", help="run every residual add as its own dfq_eltwise_q call")
    ap.add_argument("--lazy-joins", action="store_true",
                    help="take the residual adds with a single rounding (dfq_conv_q_add_lazy: the accumulator meets the second "
                         "operand at its own scale) - a different arithmetic from the default, checked against the oracle in that mode")
    ap.add_argument("--per-channel", action="store_true",
                    help="one weight format per output channel (dfq_conv_q_pc) instead of one per layer")
    ap.add_argument("--layers", action="store_true",
                    help="instead of the network pass: time the five dense layers of configs[1] on their own at --batch")
    ap.add_argument("--layer-set", choices=["config1", "3x3", "grouped", "first"], default="config1",
                    help="with --layers: the five layers of configs[1], the four 3x3 shapes of the ResNet-50-shaped network, or grouped and depthwise shapes")
    ap.add_argument("--np84", action="store_true",
                    help="the network pass on (8, 4) dynamic floating-point codes (npnet.NpPlan); with --layers: the dense layers alone (dfq_conv_np)")
    ap.add_argument("--no-np84", action="store_true", help="leave the (8, 4) pass out of the default line")
    ap.add_argument("--launch-classes", default=None,
                    help="write the per-pass order of the matrix-core launches with their roofline class (JSON) to this file")
    ap.add_argument("--no-mfma-rate", action="store_true", help="skip the register-only matrix-instruction rate probe")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three 256 MiB device copies (a kernel of known traffic, to scale HBM counters by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(the path would shard by batch, with no exchange between GPUs)", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_1805_07941_amd import binding as B
    from paper_1805_07941_amd import net as gnet
    from paper_1805_07941_amd import probe

    B.lib()
    if not torch.cuda.is_available():
        print("bench.py: needs a GPU", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.layers:
        (bench_layers_np if args.np84 else bench_layers)(args)
        return
    if args.np84:
        line = bench_net_np(args)
        print(json.dumps(line))
        pc = line["parity_checked"]
        if pc is not None and pc["images_with_identical_logits"] != pc["images"]:
            print("bench.py: the timed plan's logits differ from the oracle's", file=sys.stderr)
            sys.exit(1)
        return

    net = wl.resnet50(batch=args.batch)
    x_host = net.input_float()
    x = torch.from_numpy(x_host).to(dev)
    qz, _ = gnet.calibrate(net, x[:args.calib].contiguous(), keep_tensors=False, per_channel=args.per_channel)
    if args.lazy_joins and (args.no_fuse or args.per_channel):
        print("bench.py: --lazy-joins goes with fused joins and one weight format per layer", file=sys.stderr)
        sys.exit(2)
    plan = gnet.Plan(net, qz, args.batch, keep_all=False, fuse=not args.no_fuse, lazy_joins=args.lazy_joins)

    convs = conv_nodes(net)
    H0, W0, C0 = net.in_shape
    variant_of = {}
    for nd in convs:
        H, W, C = net.shapes[nd.srcs[0]]
        variant_of[nd.name] = B.conv_q_select(args.batch, H, W, C, nd.K, nd.R, nd.R, nd.stride, nd.pad, nd.groups)
    matrix_core = (B.CONV_MFMA, B.CONV_POINTWISE)   # the dense kernels on the int8 matrix cores
    mfma_nodes = [nd for nd in convs if variant_of[nd.name] in matrix_core]

    # instrumented pass: the plan's own call list with an event pair around each launch of the
    # matrix-core convolution kernels
    events = []
    mfma_names = {nd.name for nd in mfma_nodes}

    def run_step_recorded():
        st = B._stream(None)
        for (fn, cargs), name in zip(plan._calls_for(x), plan.call_nodes):
            mf = name in mfma_names and fn.__name__ in ("dfq_conv_q", "dfq_conv_q_add", "dfq_conv_q_pc", "dfq_conv_q_pc_add", "dfq_conv_q_add_lazy")
            if mf:
                e0, e1 = event_pool.pop(), event_pool.pop()
                e0.record()
            rc = fn(*cargs, st)
            if rc != B.OK:
                raise B.DfqError(rc, fn.__name__)
            if mf:
                e1.record()
                events.append((name, e0, e1))

    # ---- timed region: exactly K steps, bracketed by synchronize on both sides
    step = (lambda: plan.run(x)) if args.no_graph else (lambda: plan.run_graph(x))
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # ---- the same K steps again, launched call by call with an event pair around every launch of
    # the matrix-core convolution kernel (events and kernels share torch's current stream).  A
    # short spin kernel first lets the host run ahead, so that the intervals hold no launch gaps.
    record = not args.no_kernel_events
    event_pool = []
    if record:
        event_pool = [torch.cuda.Event(enable_timing=True) for _ in range(2 * len(mfma_nodes) * args.steps)]
        for _ in range(args.steps):
            torch.cuda._sleep(6_000_000)
            run_step_recorded()
        torch.cuda.synchronize()

    if args.copy_probe:
        src = torch.zeros(256 << 20, dtype=torch.int8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            B.concat_q([src.view(-1, 16)], [0], 0, out=dst.view(-1, 16))   # format-preserving concat of one branch = a copy
        torch.cuda.synchronize()
        del src, dst

    # ---- what the matrix instruction itself sustains on this chip for three kinds of operand data
    # (register-only loop, nothing else running): the ceiling under the chip's power limit
    mfma_rate = None
    if not args.no_mfma_rate:
        mid = [nd for nd in mfma_nodes if nd.R == 3 and net.shapes[nd.srcs[0]][2] == 256]
        sink = torch.empty(2048 * 512, dtype=torch.int32, device=dev)
        rnd_a = torch.randint(-128, 128, (1 << 16,), dtype=torch.int8, device=dev)
        rnd_b = torch.randint(-128, 128, (1 << 16,), dtype=torch.int8, device=dev)
        zero = torch.zeros(1 << 16, dtype=torch.int8, device=dev)
        sets = [("zeros", zero, zero), ("uniform_random_int8", rnd_a, rnd_b)]
        if mid:
            nd = mid[len(mid) // 2]
            sets.append(("network_data", qz.w[nd.name].reshape(-1), plan.buf[nd.srcs[0]].reshape(-1)))
        mfma_rate = {"unit": "TOP/s", "what": "v_mfma_i32_32x32x32_i8 in a register-only loop, 2048 workgroups of 8 wavefronts; "
                     "network_data = weights and input activations of a 3x3 layer of the pass; item_loop_* = the dense kernel's "
                     "item pipeline (matrix instructions + barrier + LDS operand reads, no global loads) on the same data"}
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for label, a_t, b_t in sets:
            for prefix, fn, n_warm, n_run in (("", probe.mfma_rate, 2000, 8000), ("item_loop_", probe.item_loop_rate, 1000, 4000)):
                fn(a_t, b_t, sink, 2048, n_warm)          # warm-up: clocks settle under this load
                e0.record()
                ops_probe = fn(a_t, b_t, sink, 2048, n_run)
                e1.record()
                torch.cuda.synchronize()
                mfma_rate[prefix + label] = round(ops_probe / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)

    n_joins = sum(1 for nd in net.nodes if nd.op == "eltwise")
    n_fused = sum(1 for fn, _ in plan._calls_for(x) if fn.__name__ in ("dfq_conv_q_add", "dfq_conv_q_pc_add", "dfq_conv_q_add_lazy"))
    macs_step = net.macs_per_image() * args.batch
    tops = 2 * macs_step / (ms_per_step * 1e-3) / 1e12
    imgs = args.batch / (ms_per_step * 1e-3)

    roofline, roofline_other = None, None
    per_layer = []
    if record and events:
        dur = {}
        for name, e0, e1 in events:
            dur.setdefault(name, []).append(e0.elapsed_time(e1))
        ops = 0.0
        tsum = 0.0
        fused_names = {name for (fn, _), name in zip(plan._calls_for(x), plan.call_nodes) if fn.__name__ in ("dfq_conv_q_add", "dfq_conv_q_pc_add", "dfq_conv_q_add_lazy")}
        # launches by what bounds them at the published peaks: ops / 5 POP/s against bytes / 8 TB/s
        layer_class = {}
        cls = {"mfma": dict(launches=0, ms=0.0, ops=0.0, bytes=0.0, roof_ms=0.0),
               "hbm": dict(launches=0, ms=0.0, ops=0.0, bytes=0.0, roof_ms=0.0)}
        for nd in mfma_nodes:
            ms = sum(dur[nd.name]) / len(dur[nd.name])
            o = 2.0 * node_macs(net, nd) * args.batch
            C = net.shapes[nd.srcs[0]][2]
            by = node_bytes(net, nd) * args.batch + nd.K * nd.R * nd.R * C + 4 * nd.K
            if nd.name in fused_names:            # the fused add reads one more tensor of the output's size
                P, Q, K = net.shapes[nd.dst]
                by += P * Q * K * args.batch
            ops += o
            tsum += ms
            t_m, t_h = o / (INT8_MFMA_PEAK_TOPS * 1e12) * 1e3, by / (HBM_PEAK_GBS * 1e9) * 1e3
            layer_class[nd.name] = "mfma" if t_m >= t_h else "hbm"
            c = cls[layer_class[nd.name]]
            c["launches"] += 1; c["ms"] += ms; c["ops"] += o; c["bytes"] += by; c["roof_ms"] += max(t_m, t_h)
            per_layer.append(dict(layer=nd.name, bound=layer_class[nd.name], us=round(ms * 1e3, 1), tops=round(o / ms / 1e9, 1),
                                  gbs=round(by / ms / 1e6, 1), min_us=round(min(dur[nd.name]) * 1e3, 1),
                                  max_us=round(max(dur[nd.name]) * 1e3, 1)))
        # HBM bytes per launch as the memory counters saw them, per class: the committed summary of two counter
        # runs of this command (FETCH_SIZE, WRITE_SIZE, each scaled by the copy probe), or null
        traffic = {"hbm": None, "mfma": None, "source": None}
        tpath = os.path.join(ROOT, "profiles", "bench_resnet50_b256_hbm_traffic.txt")
        # (the summary covers the default command only: batch 256, per-layer formats, fused joins)
        if os.path.exists(tpath) and args.batch == 256 and not args.no_fuse and not args.per_channel and not args.lazy_joins:
            import re
            txt = open(tpath).read()
            for c in ("hbm", "mfma"):
                m = re.search(r"^hbm_bytes_per_launch_%s_bound\s*=\s*([0-9.eE+]+)" % c, txt, re.M)
                traffic[c] = float(m.group(1)) if m else None
            traffic["source"] = "profiles/bench_resnet50_b256_hbm_traffic.txt (counter runs of this command; not measured by this run)"

        def cls_obj(c, label):
            d = cls[c]
            n = max(d["launches"], 1)
            if c == "mfma":
                ach, peak, unit = d["ops"] / max(d["ms"], 1e-9) / 1e9, INT8_MFMA_PEAK_TOPS, "TOP/s"
            else:
                ach, peak, unit = d["bytes"] / max(d["ms"], 1e-9) / 1e6, HBM_PEAK_GBS, "GB/s"
            return dict(bound=c, kernel=label % d["launches"], achieved=round(ach, 1), peak=peak, unit=unit,
                        frac=round(ach / peak, 4), traffic=traffic[c], traffic_source=traffic["source"],
                        launches=d["launches"], avg_launch_us=round(d["ms"] / n * 1e3, 2),
                        algorithmic_bytes_per_launch=round(d["bytes"] / n), ops_per_launch=round(d["ops"] / n),
                        share_of_step=round(d["ms"] / ms_per_step, 3))

        hbm_obj = cls_obj("hbm", "conv_pw_kernel / conv_mfma_kernel: the %d launches per step that 8 TB/s bounds before 5 POP/s does "
                                 "(1x1 layers of stages 2-4 and the joins fused into them)")
        mfma_obj = cls_obj("mfma", "conv_mfma_kernel: the %d launches per step that 5 POP/s bounds (3x3 layers, stage-5 1x1 layers, FC)")
        # `roofline` is the class that takes more of the step; the other one is carried beside it
        roofline, roofline_other = (hbm_obj, mfma_obj) if cls["hbm"]["ms"] >= cls["mfma"]["ms"] else (mfma_obj, hbm_obj)
        roofline["min_roofline_frac_all_%d_launches" % len(mfma_nodes)] = round((cls["hbm"]["roof_ms"] + cls["mfma"]["roof_ms"]) / tsum, 4)
        roofline["mfma_rate_measured"] = mfma_rate
        if args.launch_classes:
            order = []
            for (fn, _), name in zip(plan._calls_for(x), plan.call_nodes):
                if name in mfma_names and fn.__name__ in ("dfq_conv_q", "dfq_conv_q_add", "dfq_conv_q_pc", "dfq_conv_q_pc_add", "dfq_conv_q_add_lazy"):
                    order.append(dict(layer=name, bound=layer_class[name]))
            json.dump(order, open(args.launch_classes, "w"))

    # ---- outside the timed region: the oracle on a bounded sample of the same images, as the CPU baseline and
    # as the check of what was timed - the logits the timed plan produced for those images must equal the
    # oracle's exactly (the oracle calibrates for itself, so formats, weights and every layer are covered)
    cpu, parity_checked = None, None
    if args.cpu_sample > 0:
        import numpy as np
        n_cpu = min(args.cpu_sample, args.batch)
        ref_logits, cpu = cpu_baseline(net, n_cpu, min(args.calib, args.batch), per_channel=args.per_channel, lazy_joins=args.lazy_joins)
        gpu_logits = step().cpu().numpy()[:n_cpu]
        equal = int(sum(bool(np.array_equal(gpu_logits[i], ref_logits[i])) for i in range(n_cpu)))
        parity_checked = dict(images=n_cpu, images_with_identical_logits=equal, tolerance=0,
                              what="float logits of the timed plan (same launch path) against the CPU oracle's")

    line = {
        "metric": "int8 conv TOPS (2*MAC/s), whole quantized ResNet-50-shaped pass, b=%d" % args.batch,
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "launch": "per-call from Python" if args.no_graph else "HIP graph replay of the fixed call sequence",
        "joins": "each residual add its own dfq_eltwise_q call" if args.no_fuse else
                 "%d of %d residual adds run inside the convolution in front of them (%s)" % (n_fused, n_joins, "dfq_conv_q_pc_add" if args.per_channel else
                                                                                              "dfq_conv_q_add_lazy: ONE rounding per join, a different arithmetic from the default" if args.lazy_joins
                                                                                              else "dfq_conv_q_add"),
        "first_layer": {"dfq_conv_q_maxpool": "convolution and the max-pooling behind it in one kernel (dfq_conv_q_maxpool)",
                        "dfq_conv_q_pc_maxpool": "convolution and the max-pooling behind it in one kernel (dfq_conv_q_pc_maxpool)",
                        "dfq_quantize_conv_q_maxpool": "input conversion, convolution and max-pooling in one kernel (dfq_quantize_conv_q_maxpool)",
                        "dfq_quantize_conv_q_pc_maxpool": "input conversion, convolution and max-pooling in one kernel (dfq_quantize_conv_q_pc_maxpool)",
                        }.get(next((fn.__name__ for fn, _ in plan._calls_for(x) if "maxpool" in fn.__name__), None), "convolution, then dfq_pool_q"),
        "weight_formats": "one per output channel (dfq_conv_q_pc)" if args.per_channel else "one per layer",
        "config": {"workload": "configs[4]: ResNet-50-shaped int8 network, 224x224x3, batch %d, formats from a "
                               "single-batch calibrate() on %d images" % (args.batch, args.calib),
                   "global_batch": args.batch},
        "images_per_s": round(imgs, 1),
        "pct_int8_mfma_peak": round(100 * tops / INT8_MFMA_PEAK_TOPS, 2),
        "roofline": roofline,
        "roofline_other_class": roofline_other,
        "cpu_baseline": cpu,
        "parity_checked": parity_checked,
        "mfma_layers": per_layer,
    }
    # the second workload beside the headline one: the same network with every tensor on (8, 4) dynamic floating-point
    # codes (only for the default command with its oracle legs; `--np84` alone prints its full line)
    np_bad = False
    if (not args.no_np84 and args.cpu_sample > 0 and args.batch == 256 and not args.no_fuse and not args.per_channel and not args.lazy_joins and not args.no_graph):
        del plan
        torch.cuda.empty_cache()
        nl = bench_net_np(args)
        line["second_workload_np84"] = {k: nl[k] for k in ("metric", "value", "unit", "ms_per_step", "images_per_s", "dtype", "roofline", "calls",
                                                             "cpu_baseline", "parity_checked")}
        pc = nl["parity_checked"]
        np_bad = pc is not None and pc["images_with_identical_logits"] != pc["images"]
    print(json.dumps(line))
    if (parity_checked is not None and parity_checked["images_with_identical_logits"] != parity_checked["images"]) or np_bad:
        print("bench.py: the timed plan's logits differ from the oracle's", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
