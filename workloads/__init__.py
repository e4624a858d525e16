"""Seeded synthetic workloads shared by the CPU oracle and the GPU library.

This module only *describes* inputs: tensor shapes, value distributions, layer
graphs and the seeds they are drawn from.  It contains none of the quantization
scheme's arithmetic (no rounding, no format choice, no convolution): float
weights and float images are handed out as drawn, and each side converts them
with its own implementation.

The paper's experiments run GoogLeNet v1, ResNet-50 and MobileNet v1 on ImageNet
(Sec. 4); neither the images nor the trained weights are available, so tensors
with the same layer shapes and He-normal / unit-normal statistics stand in.

Every tensor is drawn from ``numpy.random.default_rng(SEED0 + 1000*config + index)``
where ``index`` counts tensors in the fixed order: input first, then per layer
(weights, bias).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

SEED0 = 180507941


def _rng(config: int, index: int) -> np.random.Generator:
    return np.random.default_rng(SEED0 + 1000 * config + index)


def out_dim(size: int, k: int, stride: int, pad: int) -> int:
    """Output extent of a window op in floor mode."""
    return (size + 2 * pad - k) // stride + 1


def int8_activations(config: int, index: int, shape, f_in: int) -> np.ndarray:
    """Raw int8 codes clip(rint(N(0,1) * 2^f_in), -128, 127).  Code -128 can occur:
    these are synthetic inputs, not tensors emitted by the scheme."""
    r = _rng(config, index)
    v = np.rint(r.standard_normal(shape, dtype=np.float32) * np.float32(2.0 ** f_in))
    return np.clip(v, -128, 127).astype(np.int8)


# --------------------------------------------------------------------------- #
# config 0: one small conv layer with every quantity given as integers          #
# --------------------------------------------------------------------------- #

def config0() -> dict:
    """1x32x32x16 input at f=4, 3x3 conv to 16 channels, weights uniform int8 at
    f=7, bias uniform in [-2^15, 2^15] at f=11, stride 1, pad 1, ReLU, f_out=4."""
    x = int8_activations(0, 0, (1, 32, 32, 16), 4)
    w = _rng(0, 1).integers(-128, 128, size=(16, 3, 3, 16), dtype=np.int64).astype(np.int8)
    b = _rng(0, 2).integers(-(2 ** 15), 2 ** 15 + 1, size=(16,), dtype=np.int64).astype(np.int32)
    return dict(x=x, w=w, b=b, f_in=4, f_w=7, f_out=4, stride=1, pad=1, groups=1, relu=1)


# --------------------------------------------------------------------------- #
# config 1: five ResNet-50-shaped dense conv layers, each run standalone        #
# --------------------------------------------------------------------------- #

#            name            H    C     K    R
RESNET_LAYER_SET = [
    ("s2_1x1_64_64",     56,  64,   64,  1),
    ("s2_3x3_64_64",     56,  64,   64,  3),
    ("s3_3x3_128_128",   28, 128,  128,  3),
    ("s4_3x3_256_256",   14, 256,  256,  3),
    ("s5_1x1_512_2048",   7, 512, 2048,  1),
]


# the four 3x3 shapes of the ResNet-50-shaped network (stride 1), drawn like the layers of config 1
RESNET_3X3_SET = [
    ("s2_3x3_64_64",     56,  64,   64,  3),
    ("s3_3x3_128_128",   28, 128,  128,  3),
    ("s4_3x3_256_256",   14, 256,  256,  3),
    ("s5_3x3_512_512",    7, 512,  512,  3),
]


# grouped and depthwise shapes (ResNeXt- and MobileNet-like), for the kernels that take layers without a dense contraction:
# (name, H, C, K, R, groups, stride)
GROUPED_SET = [
    ("g32_56_128",      56, 128,  128,  3,  32, 1),
    ("g32_28_256",      28, 256,  256,  3,  32, 1),
    ("g64_56_256_s2",   56, 256,  256,  3,  64, 2),
    ("dw_112_32",      112,  32,   32,  3,  32, 1),
    ("dw_56_128",       56, 128,  128,  3, 128, 1),
    ("dw_14_512",       14, 512,  512,  3, 512, 1),
]


# first layers of image networks (3 input channels, stride 2), same entry layout as GROUPED_SET
FIRST_LAYER_SET = [
    ("first_7x7_3_64",  224,   3,   64,  7,   1, 2),
    ("first_3x3_3_32",  224,   3,   32,  3,   1, 2),
]


def config1_layer(i: int, batch: int = 32, layer_set=None) -> dict:
    """Layer i of the set: int8 input at a per-layer f_in in {2..6}, float He-normal
    weights, float N(0, 0.1) bias; stride 1, pad R//2, ReLU.  The weight format,
    the integer bias and f_out are for each implementation to derive.
    layer_set: RESNET_LAYER_SET (config 1, the default), RESNET_3X3_SET (tensor indices from 100), GROUPED_SET (from 200,
    with groups and stride per entry) or FIRST_LAYER_SET (from 300)."""
    entry = (layer_set or RESNET_LAYER_SET)[i]
    name, H, C, K, R = entry[:5]
    groups, stride = (entry[5], entry[6]) if len(entry) > 5 else (1, 1)
    base = 10 * i + (100 if layer_set is RESNET_3X3_SET else 200 if layer_set is GROUPED_SET else 300 if layer_set is FIRST_LAYER_SET else 0)
    f_in = int(_rng(1, base + 0).integers(2, 7))
    x = int8_activations(1, base + 1, (batch, H, H, C), f_in)
    w = (_rng(1, base + 2).standard_normal((K, R, R, C // groups), dtype=np.float32)
         * np.float32(np.sqrt(2.0 / (R * R * (C // groups)))))
    b = _rng(1, base + 3).standard_normal((K,), dtype=np.float32) * np.float32(0.1)
    return dict(name=name, x=x, w_float=w, b_float=b, f_in=f_in, stride=stride, pad=R // 2,
                groups=groups, relu=1)


# --------------------------------------------------------------------------- #
# layer graphs (configs 2, 3, 4)                                                #
# --------------------------------------------------------------------------- #

@dataclass
class Node:
    """One operation of a network.  ``op`` is conv | maxpool | avgpool | eltwise |
    concat.  Tensors are named; shapes are (H, W, C) per image."""
    op: str
    name: str
    srcs: List[str]
    dst: str
    K: int = 0
    R: int = 0
    stride: int = 1
    pad: int = 0
    groups: int = 1
    relu: bool = False
    fixed_f_out: Optional[int] = None   # force the output format instead of calibrating it
    widx: int = -1                      # tensor index of this node's weights (bias = widx + 1)


@dataclass
class Net:
    config: int
    name: str
    batch: int
    in_shape: tuple                     # (H, W, C)
    nodes: List[Node] = field(default_factory=list)
    shapes: Dict[str, tuple] = field(default_factory=dict)
    input_name: str = "input"
    output_name: str = ""
    fixed_f_input: Optional[int] = None
    input_is_int8: bool = False
    f_input_codes: int = 0
    scale_layers: bool = False          # every convolution is followed by a per-channel affine layer (batch norm
                                        # in its inference form); each side folds it into the float weights itself

    # ---- construction helpers -------------------------------------------- #
    def _next_widx(self) -> int:
        n = sum(1 for nd in self.nodes if nd.op == "conv")
        return 1 + 2 * n

    def conv(self, name, src, K, R, stride=1, pad=0, groups=1, relu=True, fixed_f_out=None, dst=None):
        H, W, C = self.shapes[src]
        dst = dst or name
        nd = Node("conv", name, [src], dst, K=K, R=R, stride=stride, pad=pad, groups=groups,
                  relu=relu, fixed_f_out=fixed_f_out, widx=self._next_widx())
        self.nodes.append(nd)
        self.shapes[dst] = (out_dim(H, R, stride, pad), out_dim(W, R, stride, pad), K)
        return dst

    def pool(self, mode, name, src, k, stride, pad=0):
        H, W, C = self.shapes[src]
        self.nodes.append(Node(mode, name, [src], name, R=k, stride=stride, pad=pad))
        self.shapes[name] = (out_dim(H, k, stride, pad), out_dim(W, k, stride, pad), C)
        return name

    def eltwise(self, name, a, b, relu=True):
        assert self.shapes[a] == self.shapes[b]
        self.nodes.append(Node("eltwise", name, [a, b], name, relu=relu))
        self.shapes[name] = self.shapes[a]
        return name

    def concat(self, name, srcs, fixed_f_out=None):
        H, W, _ = self.shapes[srcs[0]]
        assert all(self.shapes[s][:2] == (H, W) for s in srcs)
        self.nodes.append(Node("concat", name, list(srcs), name, fixed_f_out=fixed_f_out))
        self.shapes[name] = (H, W, sum(self.shapes[s][2] for s in srcs))
        return name

    # ---- data -------------------------------------------------------------- #
    def input_float(self, batch: Optional[int] = None) -> np.ndarray:
        """N(0,1) float32 images, NHWC.  Image i is the same whatever the batch."""
        n = self.batch if batch is None else batch
        H, W, C = self.in_shape
        return _rng(self.config, 0).standard_normal((self.batch, H, W, C), dtype=np.float32)[:n]

    def input_int8(self) -> np.ndarray:
        H, W, C = self.in_shape
        return int8_activations(self.config, 0, (self.batch, H, W, C), self.f_input_codes)

    def weights(self, nd: Node):
        """He-normal float32 weights [K][R][R][C/groups] and N(0, 0.1) bias [K]."""
        assert nd.op == "conv"
        C = self.shapes[nd.srcs[0]][2]
        Cg = C // nd.groups
        fan_in = nd.R * nd.R * Cg
        w = (_rng(self.config, nd.widx).standard_normal((nd.K, nd.R, nd.R, Cg), dtype=np.float32)
             * np.float32(np.sqrt(2.0 / fan_in)))
        b = _rng(self.config, nd.widx + 1).standard_normal((nd.K,), dtype=np.float32) * np.float32(0.1)
        return w, b

    def scale_shift(self, nd: Node):
        """Parameters of the affine layer behind convolution nd (when the network has them): per output channel a
        scale drawn uniformly from [0.5, 1.5) and a shift drawn from N(0, 0.1), float32."""
        assert nd.op == "conv" and self.scale_layers
        r = _rng(self.config, 5000 + nd.widx)
        scale = (np.float32(0.5) + r.random((nd.K,), dtype=np.float32)).astype(np.float32)
        shift = r.standard_normal((nd.K,), dtype=np.float32) * np.float32(0.1)
        return scale, shift

    def macs_per_image(self) -> int:
        total = 0
        for nd in self.nodes:
            if nd.op == "conv":
                C = self.shapes[nd.srcs[0]][2]
                P, Q, K = self.shapes[nd.dst]
                total += P * Q * K * nd.R * nd.R * (C // nd.groups)
        return total


def inception_block(batch: int = 64, hw: int = 28) -> Net:
    """Config 2: GoogLeNet-style block on an int8 hw x hw x 256 input.  The four
    branch outputs are forced to fractional lengths drawn from {2..6} (they may
    saturate: intended) and concatenated into the coarsest of them."""
    net = Net(2, "inception", batch, (hw, hw, 256), input_is_int8=True)
    net.f_input_codes = int(_rng(2, 900).integers(2, 7))
    net.shapes["input"] = net.in_shape
    fb = [int(v) for v in _rng(2, 901).integers(2, 7, size=4)]
    b1 = net.conv("b1_1x1", "input", 64, 1, fixed_f_out=fb[0])
    t = net.conv("b2_reduce", "input", 96, 1)
    b2 = net.conv("b2_3x3", t, 128, 3, pad=1, fixed_f_out=fb[1])
    t = net.conv("b3_reduce", "input", 16, 1)
    b3 = net.conv("b3_5x5", t, 32, 5, pad=2, fixed_f_out=fb[2])
    t = net.pool("maxpool", "b4_pool", "input", 3, 1, pad=1)
    b4 = net.conv("b4_proj", t, 32, 1, fixed_f_out=fb[3])
    net.output_name = net.concat("concat", [b1, b2, b3, b4], fixed_f_out=min(fb))
    return net


def mobilenet_v1(batch: int = 128, hw: int = 224, classes: int = 1000, scale_layers: bool = False) -> Net:
    """Config 3: 3x3/2 stem to 32, 13 depthwise-separable blocks, global average
    pool, fully connected layer.  Input N(0,1) images quantized at f = 5."""
    net = Net(3, "mobilenet_v1", batch, (hw, hw, 3), fixed_f_input=5, scale_layers=scale_layers)
    net.shapes["input"] = net.in_shape
    t = net.conv("stem", "input", 32, 3, stride=2, pad=1)
    widths = [64, 128, 128, 256, 256, 512, 512, 512, 512, 512, 512, 1024, 1024]
    strides = [1, 2, 1, 2, 1, 2, 1, 1, 1, 1, 1, 2, 1]
    for i, (wd, st) in enumerate(zip(widths, strides), start=1):
        C = net.shapes[t][2]
        t = net.conv(f"dw{i}", t, C, 3, stride=st, pad=1, groups=C)
        t = net.conv(f"pw{i}", t, wd, 1)
    H = net.shapes[t][0]
    t = net.pool("avgpool", "gap", t, H, 1)
    net.output_name = net.conv("fc", t, classes, 1, relu=False)
    return net


def resnet50(batch: int = 256, hw: int = 224, classes: int = 1000, scale_layers: bool = False) -> Net:
    """Config 4: 7x7/2 stem, 3x3/2 max-pool, bottleneck stages [3,4,6,3] (stride on
    the 3x3), projection shortcut on the first block of each stage, residual
    joins with ReLU, global average pool, fully connected layer."""
    net = Net(4, "resnet50", batch, (hw, hw, 3), scale_layers=scale_layers)
    net.shapes["input"] = net.in_shape
    t = net.conv("stem", "input", 64, 7, stride=2, pad=3)
    t = net.pool("maxpool", "pool1", t, 3, 2, pad=1)
    for si, (nblk, wd) in enumerate(zip([3, 4, 6, 3], [64, 128, 256, 512]), start=2):
        for bi in range(nblk):
            st = 2 if (bi == 0 and si > 2) else 1
            pre = f"s{si}b{bi}"
            a = net.conv(pre + "_a", t, wd, 1)
            b = net.conv(pre + "_b", a, wd, 3, stride=st, pad=1)
            c = net.conv(pre + "_c", b, 4 * wd, 1, relu=False)
            sc = net.conv(pre + "_proj", t, 4 * wd, 1, stride=st, relu=False) if bi == 0 else t
            t = net.eltwise(pre + "_add", c, sc, relu=True)
    H = net.shapes[t][0]
    t = net.pool("avgpool", "gap", t, H, 1)
    net.output_name = net.conv("fc", t, classes, 1, relu=False)
    return net
