"""GPU parity on the five configurations: each side derives formats, integer weights and
biases with its own implementation from the same seeded float tensors; every int8 tensor,
every chosen format and the dequantized logits must agree exactly (tolerance 0).

Full-size runs (the launch configuration the benchmark times) are checked on the images /
output elements the oracle can afford: images are independent, so image i of a large GPU
batch must equal the oracle's result for that image alone."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle as orc
import oracle.net as onet
import workloads as wl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1805_07941_amd import binding, net
    binding.lib()
    return binding, net


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.cpu().numpy()


def _derive_layer_oracle(L):
    f_w = orc.frac_from_absmax_f32(orc.absmax_f32(L["w_float"]))
    w = orc.quantize(L["w_float"], f_w)
    b = orc.quantize_i32(L["b_float"], L["f_in"] + f_w)
    return f_w, w, b


def _derive_layer_gpu(B, L):
    wf, bf = dev(L["w_float"]), dev(L["b_float"])
    f_w = B.fmt_from_absmax_f32(float(host(B.absmax_f32(wf))[0]))
    return f_w, B.quantize(wf, f_w), B.quantize_i32(bf, L["f_in"] + f_w)


@pytest.mark.parametrize("i", range(5))
def test_config1_layers_small_batch_every_byte(G, i):
    B, _ = G
    L = wl.config1_layer(i, batch=2)
    f_w, w, b = _derive_layer_oracle(L)
    gf_w, gw, gb = _derive_layer_gpu(B, L)
    assert gf_w == f_w and np.array_equal(host(gw), w) and np.array_equal(host(gb), b)
    _, acc = orc.conv_q(L["x"], w, b, L["f_in"], f_w, 0, 1, L["pad"], 1, True, want_y=False, want_acc=True)
    f_out = orc.frac_from_absmax_i32(orc.absmax_i32(acc, relu=True), L["f_in"] + f_w)
    y = orc.requant_i32(acc, L["f_in"] + f_w - f_out, True)
    xd = dev(L["x"])
    _, gacc = B.conv_q(xd, gw, gb, L["f_in"], gf_w, 0, 1, L["pad"], 1, True, want_y=False, want_acc=True)
    gf_out = B.fmt_from_absmax_i32(B.absmax_i32_value(B.absmax_i32(gacc, relu=True)), L["f_in"] + gf_w)
    assert gf_out == f_out
    assert np.array_equal(host(gacc), acc)
    for v in (B.CONV_AUTO, B.CONV_DIRECT):
        gy, _ = B.conv_q(xd, gw, gb, L["f_in"], gf_w, gf_out, 1, L["pad"], 1, True, variant=v)
        assert np.array_equal(host(gy), y)
    assert np.abs(y).max() >= 64 and y.min() >= 0


@pytest.mark.parametrize("batch", [32, 256])
@pytest.mark.parametrize("i", range(5))
def test_config1_layers_full_size_sampled(G, i, batch):
    B, _ = G
    L = wl.config1_layer(i, batch=batch)
    f_w, w, b = _derive_layer_oracle(L)
    x = L["x"]
    N, H, W, C = x.shape
    K = w.shape[0]
    f_out = L["f_in"] + f_w - 7          # a fixed 7-bit rescale: full-size accumulators are not reduced on the CPU
    gy, gacc = B.conv_q(dev(x), dev(w), dev(b), L["f_in"], f_w, f_out, 1, L["pad"], 1, True, want_acc=True)
    gy, gacc = host(gy), host(gacc)
    rng = np.random.default_rng(1000 + i)
    pts = [(0, 0, 0, 0), (N - 1, H - 1, W - 1, K - 1), (N - 1, 0, W - 1, 0), (0, H - 1, 0, K - 1)]
    pts += [tuple(int(v) for v in (rng.integers(N), rng.integers(H), rng.integers(W), rng.integers(K))) for _ in range(400)]
    for (n, p, q, k) in pts:
        a = orc.conv_acc_at(x, w, b, 1, L["pad"], 1, n, p, q, k)
        assert int(gacc[n, p, q, k]) == a, (n, p, q, k)
        assert int(gy[n, p, q, k]) == orc.requant8(max(a, 0), 7), (n, p, q, k)
    # whole images against the oracle: the first and the last of the batch
    for n in (0, N - 1):
        y_ref, acc_ref = orc.conv_q(x[n:n + 1], w, b, L["f_in"], f_w, f_out, 1, L["pad"], 1, True, want_acc=True)
        assert np.array_equal(gy[n:n + 1], y_ref) and np.array_equal(gacc[n:n + 1], acc_ref)
    assert gy.min() >= 0 and gy.max() <= 127


@pytest.mark.parametrize("i", [1, 3, 4])
def test_config1_layers_full_size_per_channel_sampled(G, i):
    """The full-size layers (batch 256, the benchmark's launch configuration) with one weight format per output
    channel: sampled accumulators and outputs against the oracle's single-element routines, two whole images."""
    B, _ = G
    L = wl.config1_layer(i, batch=256)
    wf, bf = L["w_float"], L["b_float"]
    K = wf.shape[0]
    f_wk = np.array([orc.frac_from_absmax_f32(orc.absmax_f32(wf[k])) for k in range(K)], np.int32)
    w = np.stack([orc.quantize(wf[k], int(f_wk[k])) for k in range(K)])
    b = np.array([orc.quantize_i32(bf[k:k + 1], L["f_in"] + int(f_wk[k]))[0] for k in range(K)], np.int32)
    x = L["x"]
    N, H, W, C = x.shape
    f_out = L["f_in"] + int(f_wk.min()) - 7
    gy, gacc = B.conv_q_pc(dev(x), dev(w), dev(b), L["f_in"], dev(f_wk), f_out, 1, L["pad"], 1, True, want_acc=True)
    gy2, _ = B.conv_q_pc(dev(x), dev(w), dev(b), L["f_in"], dev(f_wk), f_out, 1, L["pad"], 1, True)      # the lean kernel
    gy, gy2, gacc = host(gy), host(gy2), host(gacc)
    assert np.array_equal(gy, gy2)
    rng = np.random.default_rng(2000 + i)
    pts = [(0, 0, 0, 0), (N - 1, H - 1, W - 1, K - 1)]
    pts += [tuple(int(v) for v in (rng.integers(N), rng.integers(H), rng.integers(W), rng.integers(K))) for _ in range(300)]
    for (n, p, q, k) in pts:
        a = orc.conv_acc_at(x, w, b, 1, L["pad"], 1, n, p, q, k)
        assert int(gacc[n, p, q, k]) == a, (n, p, q, k)
        assert int(gy[n, p, q, k]) == orc.requant8(max(a, 0), L["f_in"] + int(f_wk[k]) - f_out), (n, p, q, k)
    for n in (0, N - 1):
        y_ref, _ = orc.conv_q(x[n:n + 1], w, b, L["f_in"], f_wk, f_out, 1, L["pad"], 1, True)
        assert np.array_equal(gy[n:n + 1], y_ref)


def test_histogram_at_full_size(G):
    """The histogram of Algorithm 1 on a tensor of the benchmark's largest size (205 M accumulators)."""
    B, _ = G
    g = torch.Generator(device=DEV)
    g.manual_seed(7)
    x = (torch.randn(256 * 56 * 56 * 256, device=DEV, generator=g) * 30000).to(torch.int32)
    xh = host(x)
    counts, j, m = orc.hist_i32(xh, relu=True)
    gm = B.absmax_i32_value(B.absmax_i32(x, relu=True))
    assert gm == m
    h = host(B.hist_i32(x, j, relu=True)).view(np.uint32)
    assert np.array_equal(h[:len(counts)].astype(np.uint64), counts) and int(h.astype(np.uint64).sum()) == x.numel()
    assert B.threshold_search(h, j, m)[0] == orc.threshold_search(counts, j, m)[0]


def _compare_calibration(net, qz_o, t_o, qz_g, t_g):
    assert qz_g.frac == qz_o.frac
    assert qz_g.w_frac.keys() == qz_o.w_frac.keys()
    for name in qz_o.w_frac:
        assert np.array_equal(np.asarray(qz_g.w_frac[name]), np.asarray(qz_o.w_frac[name])), name
    for name in qz_o.w:
        assert np.array_equal(host(qz_g.w[name]), qz_o.w[name]), name
        assert np.array_equal(host(qz_g.b[name]), qz_o.b[name]), name
    for name in t_o:
        assert np.array_equal(host(t_g[name]), t_o[name]), name


def test_config2_inception_block(G):
    B, gnet = G
    net = wl.inception_block(batch=64)
    x = net.input_int8()
    calib = x[:4]
    qz_o, t_o = onet.calibrate(net, calib)
    qz_g, t_g = gnet.calibrate(net, dev(calib))
    _compare_calibration(net, qz_o, t_o, qz_g, t_g)
    # full batch on the GPU with those formats; three images checked against the oracle
    plan = gnet.Plan(net, qz_g, 64)
    plan.run(dev(x))
    out = host(plan.buf[net.output_name])
    assert out.shape == (64, 28, 28, 256)
    for i in (0, 31, 63):
        t = onet.infer(net, qz_o, x[i:i + 1])
        for name in t:
            if name != net.input_name:
                assert np.array_equal(host(plan.buf[name][i:i + 1]), t[name]), (i, name)
    assert int(np.abs(out).max()) > 0 and int(out.min()) >= 0      # every branch ends in a ReLU


@pytest.mark.parametrize("match_joins", [False, True], ids=["rescaling_concat", "matched_join_scales"])
def test_config2_branches_written_into_the_joined_tensor(G, match_joins):
    """Plan(fuse=True): a branch convolution whose format is the concat's writes straight into its channel slice (row
    pitch of the joined tensor); with match_joins calibration (Sec. 3: input scales of a join are matched) that holds
    for every branch and no concat kernel runs.  Formats, tensors and the joined output against the oracle."""
    B, gnet = G
    net = wl.inception_block(batch=64)
    x = net.input_int8()
    calib = x[:4]
    qz_o, t_o = onet.calibrate(net, calib, match_joins=match_joins)
    qz_g, t_g = gnet.calibrate(net, dev(calib), match_joins=match_joins)
    _compare_calibration(net, qz_o, t_o, qz_g, t_g)
    cat = net.nodes[-1]
    if match_joins:
        assert all(qz_o.frac[s] == qz_o.frac[cat.dst] for s in cat.srcs)
    for keep_all in (True, False):
        plan = gnet.Plan(net, qz_g, 64, keep_all=keep_all, fuse=True)
        n_direct = len(plan.slice_of)
        assert n_direct == (4 if match_joins else sum(1 for s in cat.srcs if qz_o.frac[s] == qz_o.frac[cat.dst])) and n_direct >= 1
        for rep in range(2):
            plan.buf[cat.dst].fill_(55)
            plan.run_graph(dev(x)) if rep else plan.run(dev(x))
            out = host(plan.buf[net.output_name])
            for i in (0, 17, 63):
                t = onet.infer(net, qz_o, x[i:i + 1])
                assert np.array_equal(out[i:i + 1], t[net.output_name]), (keep_all, rep, i)
                for name in plan.resident():
                    if name != net.input_name:
                        assert np.array_equal(host(plan.buf[name][i:i + 1]), t[name]), (i, name)
        n_concat = sum(1 for fn, _ in plan._calls if fn.__name__.startswith("dfq_concat_q"))
        assert n_concat == (0 if match_joins else 1) or n_direct < 4


@pytest.mark.parametrize("which", ["mobilenet_v1", "resnet50"])
def test_config3_and_4_networks(G, which):
    B, gnet = G
    batch = 128 if which == "mobilenet_v1" else 256
    net = getattr(wl, which)(batch=batch)
    x = net.input_float()
    calib = x[:2]                          # a small single calibration batch keeps the oracle to seconds
    qz_o, t_o = onet.calibrate(net, calib)
    qz_g, t_g = gnet.calibrate(net, dev(calib))
    _compare_calibration(net, qz_o, t_o, qz_g, t_g)
    del t_g
    plan = gnet.Plan(net, qz_g, batch)
    logits = host(plan.run(dev(x))).copy()
    assert logits.shape == (batch, 1000) and np.isfinite(logits).all()
    for i in (1, batch - 1):
        t = onet.infer(net, qz_o, x[i:i + 1])
        for name in t:
            assert np.array_equal(host(plan.buf[name][i:i + 1]), t[name]), (i, name)
        ref = onet.logits(net, qz_o, t)
        assert np.array_equal(logits[i:i + 1], ref)        # absolute tolerance 0
    # pooled buffers (the benchmark's memory plan) give the same logits
    plan2 = gnet.Plan(net, qz_g, batch, keep_all=False)
    assert np.array_equal(host(plan2.run(dev(x))), logits)
    assert np.abs(logits).max() > 0
    del plan, plan2
    _check_benchmark_plan(gnet, net, qz_g, qz_o, x, logits, batch, min_fused=16 if which == "resnet50" else 0)


def _check_benchmark_plan(gnet, net, qz_g, qz_o, x, logits_unfused, batch, min_fused=0):
    """The plan exactly as bench.py builds and times it - pooled buffers, joins fused into the convolutions in front of
    them, replayed from a HIP graph, at the full batch: logits of the whole batch against the unfused plan's (when
    given), and for three images the logits and every tensor still resident after the pass against the oracle."""
    xd = dev(x)
    plan = gnet.Plan(net, qz_g, batch, keep_all=False, fuse=True)
    for rep in range(2):                                  # the capture run and one replay
        got = host(plan.run_graph(xd)).copy()
        if logits_unfused is not None:
            assert np.array_equal(got, logits_unfused), rep
    n_fused = sum(1 for fn, _ in plan._calls if fn.__name__ in ("dfq_conv_q_add", "dfq_conv_q_pc_add"))
    assert n_fused >= min_fused, n_fused
    names = plan.resident()
    assert net.output_name in names
    for i in (0, batch // 2 + 1, batch - 1):
        t = onet.infer(net, qz_o, x[i:i + 1])
        assert np.array_equal(got[i:i + 1], onet.logits(net, qz_o, t)), i          # absolute tolerance 0
        for name in names:
            if name != net.input_name or not net.input_is_int8:
                assert np.array_equal(host(plan.buf[name][i:i + 1]), t[name]), (i, name)
    return n_fused


def test_resnet50_benchmark_plan_per_channel_full_batch(G):
    """bench.py --per-channel: the ResNet-50-shaped network at batch 256 with one weight format per output channel,
    pooled buffers, fused joins, graph replay."""
    B, gnet = G
    net = wl.resnet50(batch=256)
    x = net.input_float()
    calib = x[:2]
    qz_o, t_o = onet.calibrate(net, calib, per_channel=True)
    qz_g, t_g = gnet.calibrate(net, dev(calib), per_channel=True, keep_tensors=False)
    assert qz_g.frac == qz_o.frac
    for name in qz_o.w:
        assert np.array_equal(host(qz_g.w[name]), qz_o.w[name]) and np.array_equal(host(qz_g.b[name]), qz_o.b[name]), name
        assert np.array_equal(np.asarray(qz_g.w_frac[name]), np.asarray(qz_o.w_frac[name])), name
    del t_o, t_g
    _check_benchmark_plan(gnet, net, qz_g, qz_o, x, None, 256, min_fused=16)


@pytest.mark.parametrize("which", ["mobilenet_v1", "resnet50"])
def test_per_channel_weight_formats_networks(G, which):
    """One weight format per output channel (Sec. 3): calibration and inference agree with the oracle
    in every format, weight, bias, int8 tensor and logit."""
    B, gnet = G
    batch = 16
    net = getattr(wl, which)(batch=batch, hw=96, classes=100)
    x = net.input_float()
    calib = x[:2]
    qz_o, t_o = onet.calibrate(net, calib, per_channel=True)
    qz_g, t_g = gnet.calibrate(net, dev(calib), per_channel=True)
    _compare_calibration(net, qz_o, t_o, qz_g, t_g)
    assert any(len(set(np.asarray(v).tolist())) > 1 for v in qz_o.w_frac.values())     # the formats do differ by channel
    del t_g
    for kw in (dict(), dict(keep_all=False, fuse=True)):
        plan = gnet.Plan(net, qz_g, batch, **kw)
        logits = host(plan.run(dev(x))).copy()
        for i in (0, batch - 1):
            t = onet.infer(net, qz_o, x[i:i + 1])
            assert np.array_equal(logits[i:i + 1], onet.logits(net, qz_o, t))
            if not kw:
                for name in t:
                    assert np.array_equal(host(plan.buf[name][i:i + 1]), t[name]), (i, name)
        assert np.array_equal(host(plan.run_graph(dev(x))), logits)
        if kw and which == "resnet50":
            assert sum(1 for fn, _ in plan._calls if fn.__name__ == "dfq_conv_q_pc_add") >= 4


def test_network_with_scale_layers_folded(G):
    """A ResNet-50-shaped network with an affine layer behind every convolution: both sides fold it into the float weights
    with their own code before quantizing; formats, integer weights, tensors and logits agree."""
    B, gnet = G
    net = wl.resnet50(batch=8, hw=64, classes=100, scale_layers=True)
    x = net.input_float()
    calib = x[:2]
    qz_o, t_o = onet.calibrate(net, calib)
    qz_g, t_g = gnet.calibrate(net, dev(calib))
    _compare_calibration(net, qz_o, t_o, qz_g, t_g)
    plan = gnet.Plan(net, qz_g, 8, keep_all=False, fuse=True)
    logits = host(plan.run(dev(x)))
    for i in (0, 7):
        t = onet.infer(net, qz_o, x[i:i + 1])
        assert np.array_equal(logits[i:i + 1], onet.logits(net, qz_o, t))


def test_threshold_search_calibration_network(G):
    """Calibration with Algorithm 1 as the threshold rule: same formats, weights and tensors as the oracle."""
    B, gnet = G
    net = wl.resnet50(batch=8, hw=64, classes=100)
    x = net.input_float()
    calib = x[:2]
    qz_o, t_o = onet.calibrate(net, calib, rule="search")
    qz_g, t_g = gnet.calibrate(net, dev(calib), rule="search")
    _compare_calibration(net, qz_o, t_o, qz_g, t_g)
    qz_m, _ = onet.calibrate(net, calib)
    assert qz_o.frac != qz_m.frac                      # the rule does change some formats on this input
    plan = gnet.Plan(net, qz_g, 8, keep_all=False, fuse=True)
    logits = host(plan.run(dev(x)))
    for i in (0, 7):
        t = onet.infer(net, qz_o, x[i:i + 1])
        assert np.array_equal(logits[i:i + 1], onet.logits(net, qz_o, t))


def test_fused_joins_give_the_same_logits(G):
    """A plan that runs each residual add inside the convolution in front of it must reproduce the
    unfused plan bit for bit (and through it the oracle, which the test above pins)."""
    B, gnet = G
    net = wl.resnet50(batch=16, hw=96, classes=100)
    x = dev(net.input_float())
    qz, _ = gnet.calibrate(net, x[:4].contiguous(), keep_tensors=False)
    plain = gnet.Plan(net, qz, 16)
    fused = gnet.Plan(net, qz, 16, fuse=True)
    ref = host(plain.run(x)).copy()
    got = host(fused.run(x)).copy()
    assert sum(1 for j in fused.fused.values() if net.nodes[j].op == "eltwise") == 16
    # the first layer and the max-pooling behind it run as one call too
    assert sum(1 for j in fused.fused.values() if net.nodes[j].op == "maxpool") == 1
    # ... and, the images being float, so does their conversion: no dfq_quantize call is left
    assert sum(1 for fn, _ in fused._calls if fn.__name__ == "dfq_quantize_conv_q_maxpool") == 1
    assert not any(fn.__name__ == "dfq_quantize" for fn, _ in fused._calls)
    assert net.input_name not in fused.resident()
    # first blocks of the later stages list (c, projection, add): only c fits the fused kernel, so the plan
    # runs the projection first and c together with the add
    assert fused.order != sorted(fused.order) and sorted(fused.order) == list(range(len(net.nodes)))
    n_fused = sum(1 for fn, _ in fused._calls if fn.__name__ == "dfq_conv_q_add")
    assert n_fused >= 4                              # joins behind pointwise layers with C <= 256 and a rounding step left
    assert np.array_equal(got, ref) and np.abs(ref).max() > 0
    # the add's output tensors agree as well
    for i, j in fused.fused.items():
        name = net.nodes[j].dst
        assert np.array_equal(host(fused.buf[name]), host(plain.buf[name])), name
    # pooled buffers, replayed from a graph
    pooled = gnet.Plan(net, qz, 16, keep_all=False, fuse=True)
    assert np.array_equal(host(pooled.run(x)), ref)
    assert np.array_equal(host(pooled.run_graph(x)), ref)


def test_graph_replay_matches_eager(G):
    """The captured call sequence must give the eager result on every replay, with eager work
    and synchronizations in between."""
    B, gnet = G
    net = wl.resnet50(batch=8, hw=64, classes=100)
    x = dev(net.input_float())
    qz, _ = gnet.calibrate(net, x[:4].contiguous(), keep_tensors=False)
    plan = gnet.Plan(net, qz, 8, keep_all=False)
    eager = host(plan.run(x)).copy()
    torch.cuda.synchronize()
    for i in range(4):
        plan.logits.zero_()
        got = host(plan.run_graph(x))
        assert np.array_equal(got, eager), i
        # unrelated eager work between replays
        y = B.quantize(x, 3)
        torch.cuda.synchronize()
        assert np.array_equal(host(plan.run(x)), eager)
    x2 = dev(net.input_float()[::-1].copy())
    e2 = host(plan.run(x2)).copy()
    assert np.array_equal(host(plan.run_graph(x2)), e2) and not np.array_equal(e2, eager)


def test_resnet50_lazy_joins_full_batch(G):
    """bench.py --lazy-joins: the ResNet-50-shaped network at batch 256 with all sixteen joins taken with a single
    rounding (dfq_conv_q_add_lazy), pooled buffers, graph replay: logits and every resident tensor of three images
    against the oracle's inference in the same mode; the formats are those of the ordinary calibration."""
    B, gnet = G
    batch = 256
    net = wl.resnet50(batch=batch)
    x = net.input_float()
    calib = x[:2]
    qz_o, t_o = onet.calibrate(net, calib)
    qz_g, t_g = gnet.calibrate(net, dev(calib), keep_tensors=False)
    assert qz_g.frac == qz_o.frac
    del t_o, t_g
    xd = dev(x)
    plan = gnet.Plan(net, qz_g, batch, keep_all=False, fuse=True, lazy_joins=True)
    for rep in range(2):
        got = host(plan.run_graph(xd)).copy()
    assert sum(1 for fn, _ in plan._calls if fn.__name__ == "dfq_conv_q_add_lazy") == 16
    assert not any(fn.__name__ in ("dfq_conv_q_add", "dfq_eltwise_q") for fn, _ in plan._calls)
    names = plan.resident()
    differs = 0
    for i in (0, batch // 2 + 1, batch - 1):
        t = onet.infer(net, qz_o, x[i:i + 1], lazy_joins=True)
        assert np.array_equal(got[i:i + 1], onet.logits(net, qz_o, t)), i
        for name in names:
            if name != net.input_name or not net.input_is_int8:
                assert np.array_equal(host(plan.buf[name][i:i + 1]), t[name]), (i, name)
        differs += int(not np.array_equal(onet.logits(net, qz_o, onet.infer(net, qz_o, x[i:i + 1])), got[i:i + 1]))
    assert differs > 0                         # it is a different arithmetic from the two-rounding joins
    with pytest.raises(ValueError):
        gnet.Plan(net, qz_g, batch, lazy_joins=True)
