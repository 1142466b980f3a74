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
    kind: str = "maxpool"


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


def _maxpool(net, name, src, R, stride, pad):
    s = net.tensors[src]
    Ho = out_extent(s.H, R, stride, pad)
    Wo = out_extent(s.W, R, stride, pad)
    dst = net.tensor(name, Ho, Wo, s.C)
    net.ops.append(PoolSpec(name, src, dst, R, R, stride, pad))
    return dst


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


def resnet50(image=224):
    """Config 3: the 53 convolutions of ResNet-50 (stride 2 on the first 1x1 of a stage)."""
    net = Network("resnet50", "image")
    net.tensor("image", image, image, 3)
    t = _conv(net, "conv1", "image", 64, 7, 7, stride=2, pad_h=3, pad_w=3)
    t = _maxpool(net, "pool1", t, 3, 2, 1)
    stages = [(2, 3, 64, 256), (3, 4, 128, 512), (4, 6, 256, 1024), (5, 3, 512, 2048)]
    for stage, blocks, mid, out in stages:
        for blk in range(blocks):
            tag = f"res{stage}{chr(ord('a') + blk)}"
            stride = 2 if (blk == 0 and stage > 2) else 1
            if blk == 0:
                short = _conv(net, tag + "_branch1", t, out, 1, 1, stride=stride, relu=False)
            else:
                short = t
            a = _conv(net, tag + "_branch2a", t, mid, 1, 1, stride=stride)
            b = _conv(net, tag + "_branch2b", a, mid, 3, 3)
            t = _conv(net, tag + "_branch2c", b, out, 1, 1, relu=True, res=short)
    net.outputs = [t]
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
}
