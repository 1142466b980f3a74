"""Seeded synthetic inputs and layer lists for the benchmark configurations.

This module holds no arithmetic of the method: it only draws random fp32 tensors with the
documented distributions and describes network graphs (which convolution reads which
tensor).  Both the CPU oracle's tests and the GPU path take their inputs from here, so they
see identical bits.  It imports neither of them.

Stand-ins: the paper measures throughput on "fake random data" and calibrates on
ImageNet / VOC, which are not available; N(0,1) pixels and He-normal weights with random
BatchNorm statistics take their place.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

SEED_ROOT = (1805, 8691)


def rng_for(*path):
    """Independent generator for one tensor; ``path`` = (config id, layer index, tensor tag...)."""
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(SEED_ROOT + tuple(path))))


# ------------------------------------------------------------------------------------------
# graph description
# ------------------------------------------------------------------------------------------
@dataclass
class TensorSpec:
    name: str
    H: int
    W: int
    C: int


@dataclass
class ConvSpec:
    name: str
    src: str
    dst: str
    C: int
    K: int
    R: int
    S: int
    stride: int = 1
    pad_h: int = 0
    pad_w: int = 0
    dil: int = 1
    relu: bool = True
    res: Optional[str] = None      # tensor added before the ReLU (fused element-wise sum)
    dst_c_off: int = 0             # channel offset inside dst (branch of a concat)
    kind: str = "conv"


@dataclass
class PoolSpec:
    name: str
    src: str
    dst: str
    R: int
    S: int
    stride: int
    pad: int
    mode: str = "max"              # "max" or "avg" (mean over R*S, padding counted as zeros)
    dst_c_off: int = 0             # channel offset inside dst (pooled branch of a concat)
    kind: str = "pool"


@dataclass
class Network:
    name: str
    input: str
    tensors: Dict[str, TensorSpec] = field(default_factory=dict)
    ops: List[object] = field(default_factory=list)
    outputs: List[str] = field(default_factory=list)

    def tensor(self, name, H, W, C):
        self.tensors[name] = TensorSpec(name, H, W, C)
        return name

    def convs(self):
        return [o for o in self.ops if o.kind == "conv"]

    def macs_per_image(self):
        tot = 0
        for o in self.convs():
            t = self.tensors[o.dst]
            tot += t.H * t.W * o.K * o.C * o.R * o.S
        return tot


def out_extent(n, k, stride, pad, dil=1):
    return (n + 2 * pad - dil * (k - 1) - 1) // stride + 1


def _conv(net, name, src, K, R, S, stride=1, pad_h=None, pad_w=None, dil=1, relu=True, res=None,
          dst=None, dst_c_off=0):
    s = net.tensors[src]
    if pad_h is None:
        pad_h = dil * (R - 1) // 2
    if pad_w is None:
        pad_w = dil * (S - 1) // 2
    Ho = out_extent(s.H, R, stride, pad_h, dil)
    Wo = out_extent(s.W, S, stride, pad_w, dil)
    if dst is None:
        dst = net.tensor(name, Ho, Wo, K)
    else:
        d = net.tensors[dst]
        assert (d.H, d.W) == (Ho, Wo) and dst_c_off + K <= d.C
    net.ops.append(ConvSpec(name, src, dst, s.C, K, R, S, stride, pad_h, pad_w, dil, relu, res,
                            dst_c_off))
    return dst


def _pool(net, name, src, R, stride, pad, mode="max", ceil=False, dst=None, dst_c_off=0):
    s = net.tensors[src]
    if ceil:
        Ho = -((s.H + 2 * pad - R) // -stride) + 1
        Wo = -((s.W + 2 * pad - R) // -stride) + 1
    else:
        Ho = out_extent(s.H, R, stride, pad)
        Wo = out_extent(s.W, R, stride, pad)
    if dst is None:
        dst = net.tensor(name, Ho, Wo, s.C)
    else:
        d = net.tensors[dst]
        assert (d.H, d.W) == (Ho, Wo) and dst_c_off + s.C <= d.C
    net.ops.append(PoolSpec(name, src, dst, R, R, stride, pad, mode, dst_c_off))
    return dst


def _maxpool(net, name, src, R, stride, pad):
    return _pool(net, name, src, R, stride, pad)


def single_conv3x3():
    """Config 1: one 3x3 convolution, 56x56x64 -> 64, stride 1, pad 1, fused ReLU."""
    net = Network("single_conv3x3", "x")
    net.tensor("x", 56, 56, 64)
    out = _conv(net, "conv", "x", 64, 3, 3)
    net.outputs = [out]
    return net


def bottleneck_block(H=56, C=256, mid=64):
    """Config 2: ResNet-50 bottleneck with identity shortcut (1x1, 3x3, 1x1 + sum + ReLU)."""
    net = Network("bottleneck_block", "x")
    net.tensor("x", H, H, C)
    a = _conv(net, "branch2a", "x", mid, 1, 1)
    b = _conv(net, "branch2b", a, mid, 3, 3)
    c = _conv(net, "branch2c", b, C, 1, 1, relu=True, res="x")
    net.outputs = [c]
    return net


def resnet50(image=224, sparsity_removal=False):
    """Config 3: the 53 convolutions of ResNet-50 (stride 2 on the first 1x1 of a stage).

    ``sparsity_removal`` applies the paper's graph transformation ("Model Optimization",
    the sparsity figure): the two stride-2 1x1 convolutions that open a stage read only
    every other pixel of their input, so the layer producing that input (the previous
    block's last 1x1) is given the stride 2 instead and produces only the pixels that are
    read, a 1x1 stride-2 pooling on the skip branch subsamples its residual to match, and the
    two consumers become stride 1.  Same values at the kept positions, less work."""
    net = Network("resnet50_sparse" if sparsity_removal else "resnet50", "image")
    net.tensor("image", image, image, 3)
    t = _conv(net, "conv1", "image", 64, 7, 7, stride=2, pad_h=3, pad_w=3)
    t = _maxpool(net, "pool1", t, 3, 2, 1)
    stages = [(2, 3, 64, 256), (3, 4, 128, 512), (4, 6, 256, 1024), (5, 3, 512, 2048)]
    pre_strided = False          # t already holds only the pixels a stride-2 consumer reads
    for si, (stage, blocks, mid, out) in enumerate(stages):
        for blk in range(blocks):
            tag = f"res{stage}{chr(ord('a') + blk)}"
            stride = 2 if (blk == 0 and stage > 2 and not pre_strided) else 1
            pre_strided = False
            if blk == 0:
                short = _conv(net, tag + "_branch1", t, out, 1, 1, stride=stride, relu=False)
            else:
                short = t
            a = _conv(net, tag + "_branch2a", t, mid, 1, 1, stride=stride)
            b = _conv(net, tag + "_branch2b", a, mid, 3, 3)
            last = blk == blocks - 1 and si + 1 < len(stages)
            if sparsity_removal and last:
                short = _pool(net, tag + "_skip_pool", short, 1, 2, 0)
                t = _conv(net, tag + "_branch2c", b, out, 1, 1, stride=2, relu=True, res=short)
                pre_strided = True
            else:
                t = _conv(net, tag + "_branch2c", b, out, 1, 1, relu=True, res=short)
    net.outputs = [t]
    return net


def inception_v3(image=299):
    """Config 4: the 94 convolutions of Inception-v3 (1x1, 3x3, 5x5, 1x7/7x1, 1x3/3x1,
    stride-2 reductions); the branches of a block write channel slices of one concat tensor."""
    net = Network("inception_v3", "image")
    net.tensor("image", image, image, 3)
    t = _conv(net, "conv1a", "image", 32, 3, 3, stride=2, pad_h=0, pad_w=0)
    t = _conv(net, "conv2a", t, 32, 3, 3, pad_h=0, pad_w=0)
    t = _conv(net, "conv2b", t, 64, 3, 3)
    t = _pool(net, "pool1", t, 3, 2, 0)
    t = _conv(net, "conv3b", t, 80, 1, 1)
    t = _conv(net, "conv4a", t, 192, 3, 3, pad_h=0, pad_w=0)
    t = _pool(net, "pool2", t, 3, 2, 0)

    def concat(name, src, width):
        s = net.tensors[src]
        return net.tensor(name, s.H, s.W, width)

    for i, pf in enumerate((32, 64, 64)):                       # 35 x 35
        n = f"mixed5{'bcd'[i]}"
        out = concat(n, t, 64 + 64 + 96 + pf)
        _conv(net, n + "_1x1", t, 64, 1, 1, dst=out, dst_c_off=0)
        a = _conv(net, n + "_5x5a", t, 48, 1, 1)
        _conv(net, n + "_5x5b", a, 64, 5, 5, dst=out, dst_c_off=64)
        a = _conv(net, n + "_dbla", t, 64, 1, 1)
        a = _conv(net, n + "_dblb", a, 96, 3, 3)
        _conv(net, n + "_dblc", a, 96, 3, 3, dst=out, dst_c_off=128)
        a = _pool(net, n + "_pool", t, 3, 1, 1, mode="avg")
        _conv(net, n + "_poolproj", a, pf, 1, 1, dst=out, dst_c_off=224)
        t = out
    s = net.tensors[t]
    out = net.tensor("mixed6a", out_extent(s.H, 3, 2, 0), out_extent(s.W, 3, 2, 0), 384 + 96 + 288)
    _conv(net, "mixed6a_3x3", t, 384, 3, 3, stride=2, pad_h=0, pad_w=0, dst=out, dst_c_off=0)
    a = _conv(net, "mixed6a_dbla", t, 64, 1, 1)
    a = _conv(net, "mixed6a_dblb", a, 96, 3, 3)
    _conv(net, "mixed6a_dblc", a, 96, 3, 3, stride=2, pad_h=0, pad_w=0, dst=out, dst_c_off=384)
    _pool(net, "mixed6a_pool", t, 3, 2, 0, dst=out, dst_c_off=480)
    t = out
    for i, c7 in enumerate((128, 160, 160, 192)):               # 17 x 17
        n = f"mixed6{'bcde'[i]}"
        out = concat(n, t, 768)
        _conv(net, n + "_1x1", t, 192, 1, 1, dst=out, dst_c_off=0)
        a = _conv(net, n + "_7a", t, c7, 1, 1)
        a = _conv(net, n + "_7b", a, c7, 1, 7)
        _conv(net, n + "_7c", a, 192, 7, 1, dst=out, dst_c_off=192)
        a = _conv(net, n + "_77a", t, c7, 1, 1)
        a = _conv(net, n + "_77b", a, c7, 7, 1)
        a = _conv(net, n + "_77c", a, c7, 1, 7)
        a = _conv(net, n + "_77d", a, c7, 7, 1)
        _conv(net, n + "_77e", a, 192, 1, 7, dst=out, dst_c_off=384)
        a = _pool(net, n + "_pool", t, 3, 1, 1, mode="avg")
        _conv(net, n + "_poolproj", a, 192, 1, 1, dst=out, dst_c_off=576)
        t = out
    s = net.tensors[t]
    out = net.tensor("mixed7a", out_extent(s.H, 3, 2, 0), out_extent(s.W, 3, 2, 0), 320 + 192 + 768)
    a = _conv(net, "mixed7a_3a", t, 192, 1, 1)
    _conv(net, "mixed7a_3b", a, 320, 3, 3, stride=2, pad_h=0, pad_w=0, dst=out, dst_c_off=0)
    a = _conv(net, "mixed7a_7a", t, 192, 1, 1)
    a = _conv(net, "mixed7a_7b", a, 192, 1, 7)
    a = _conv(net, "mixed7a_7c", a, 192, 7, 1)
    _conv(net, "mixed7a_7d", a, 192, 3, 3, stride=2, pad_h=0, pad_w=0, dst=out, dst_c_off=320)
    _pool(net, "mixed7a_pool", t, 3, 2, 0, dst=out, dst_c_off=512)
    t = out
    for i in range(2):                                          # 8 x 8
        n = f"mixed7{'bc'[i]}"
        out = concat(n, t, 320 + 768 + 768 + 192)
        _conv(net, n + "_1x1", t, 320, 1, 1, dst=out, dst_c_off=0)
        a = _conv(net, n + "_3a", t, 384, 1, 1)
        _conv(net, n + "_3b1", a, 384, 1, 3, dst=out, dst_c_off=320)
        _conv(net, n + "_3b2", a, 384, 3, 1, dst=out, dst_c_off=704)
        a = _conv(net, n + "_d3a", t, 448, 1, 1)
        a = _conv(net, n + "_d3b", a, 384, 3, 3)
        _conv(net, n + "_d3c1", a, 384, 1, 3, dst=out, dst_c_off=1088)
        _conv(net, n + "_d3c2", a, 384, 3, 1, dst=out, dst_c_off=1472)
        a = _pool(net, n + "_pool", t, 3, 1, 1, mode="avg")
        _conv(net, n + "_poolproj", a, 192, 1, 1, dst=out, dst_c_off=1856)
        t = out
    net.outputs = [t]
    return net


def ssd300_vgg16(image=300, classes=21):
    """Config 5: SSD-300 backbone (VGG-16 with a dilated fc6), extra layers and the 3x3
    multibox heads on six feature maps (location 4a and confidence classes*a channels)."""
    net = Network("ssd300_vgg16", "image")
    net.tensor("image", image, image, 3)
    t = "image"
    plan = [(64, 2), (128, 2), (256, 3), (512, 3), (512, 3)]
    for b, (k, n) in enumerate(plan, 1):
        for i in range(1, n + 1):
            t = _conv(net, f"conv{b}_{i}", t, k, 3, 3)
        if b == 4:
            conv4_3 = t
        if b < 5:
            t = _pool(net, f"pool{b}", t, 2, 2, 0, ceil=(b == 3))
        else:
            t = _pool(net, "pool5", t, 3, 1, 1)
    t = _conv(net, "fc6", t, 1024, 3, 3, dil=6)
    fc7 = t = _conv(net, "fc7", t, 1024, 1, 1)
    t = _conv(net, "conv6_1", t, 256, 1, 1)
    c6 = t = _conv(net, "conv6_2", t, 512, 3, 3, stride=2)
    t = _conv(net, "conv7_1", t, 128, 1, 1)
    c7 = t = _conv(net, "conv7_2", t, 256, 3, 3, stride=2)
    t = _conv(net, "conv8_1", t, 128, 1, 1)
    c8 = t = _conv(net, "conv8_2", t, 256, 3, 3, pad_h=0, pad_w=0)
    t = _conv(net, "conv9_1", t, 128, 1, 1)
    c9 = t = _conv(net, "conv9_2", t, 256, 3, 3, pad_h=0, pad_w=0)
    for src, anchors in ((conv4_3, 4), (fc7, 6), (c6, 6), (c7, 6), (c8, 4), (c9, 4)):
        net.outputs.append(_conv(net, src + "_loc", src, 4 * anchors, 3, 3, relu=False))
        net.outputs.append(_conv(net, src + "_conf", src, classes * anchors, 3, 3, relu=False))
    return net


# ------------------------------------------------------------------------------------------
# seeded parameters and inputs
# ------------------------------------------------------------------------------------------
def conv_params(config_id, layer_index, spec):
    """fp32 parameters of one conv + BatchNorm: He-normal W (KRSC), b ~ N(0, .1),
    gamma ~ U(.5, 1.5), beta ~ N(0, .1), mu ~ N(0, .1), var ~ U(.5, 1.5)."""
    g = rng_for(config_id, layer_index)
    fan_in = spec.R * spec.S * spec.C
    f32 = np.float32
    return dict(
        W=(g.standard_normal((spec.K, spec.R, spec.S, spec.C)) * np.sqrt(2.0 / fan_in)).astype(f32),
        b=(g.standard_normal(spec.K) * 0.1).astype(f32),
        gamma=g.uniform(0.5, 1.5, spec.K).astype(f32),
        beta=(g.standard_normal(spec.K) * 0.1).astype(f32),
        mu=(g.standard_normal(spec.K) * 0.1).astype(f32),
        var=g.uniform(0.5, 1.5, spec.K).astype(f32),
        eps=1e-5,
    )


def input_batch(config_id, net, batch, index=0, relu=False):
    """fp32 NHWC input batch number ``index``: N(0,1), or max(N(0,1), 0) when ``relu``."""
    t = net.tensors[net.input]
    g = rng_for(config_id, 10**6 + index)
    x = g.standard_normal((batch, t.H, t.W, t.C), dtype=np.float32)
    if relu:
        np.maximum(x, 0, out=x)
    return x


CONFIGS = {
    1: dict(make=single_conv3x3, batch=1, relu_input=True),
    2: dict(make=bottleneck_block, batch=32, relu_input=True),
    3: dict(make=resnet50, batch=64, relu_input=False),
    4: dict(make=inception_v3, batch=64, relu_input=False),
    5: dict(make=ssd300_vgg16, batch=64, relu_input=False),
    # config 3 after the paper's sparsity-removal graph transformation (not a BASELINE config)
    6: dict(make=lambda: resnet50(sparsity_removal=True), batch=64, relu_input=False),
}
