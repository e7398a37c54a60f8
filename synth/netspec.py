"""Network specifications (flat layer records) and the seeded recipe for
parameters and minibatches.

A network is a list of layer records in execution order.  `in0`/`in1` name the
producing layer (index into the list); -1 is the network input.  The same
records are handed to the CPU oracle and to the HIP library; each derives
tensor shapes on its own.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

from .rng import normal, labels_uniform, splitmix64

CONV, BN, RELU, ADD, MAXPOOL, GAP, FC, SOFTMAX_CE, BIAS = range(9)
KIND_NAMES = ["conv", "bn", "relu", "add", "maxpool", "gap", "fc", "softmax_ce", "bias"]


@dataclass
class Layer:
    kind: int
    in0: int = -1
    in1: int = -1
    cin: int = 0
    cout: int = 0
    r: int = 0
    s: int = 0
    stride: int = 1
    pad: int = 0

    def as_tuple(self) -> Tuple[int, ...]:
        return (self.kind, self.in0, self.in1, self.cin, self.cout,
                self.r, self.s, self.stride, self.pad)


@dataclass
class NetSpec:
    name: str
    in_c: int
    in_h: int
    in_w: int
    classes: int
    layers: List[Layer] = field(default_factory=list)

    def add(self, layer: Layer) -> int:
        self.layers.append(layer)
        return len(self.layers) - 1

    def as_array(self) -> np.ndarray:
        """int32 [n, 9] array with the C record layout (kind,in0,in1,cin,cout,r,s,stride,pad)."""
        return np.array([l.as_tuple() for l in self.layers], dtype=np.int32)

    def param_sizes(self) -> List[int]:
        out = []
        for l in self.layers:
            if l.kind == CONV:
                out.append(l.cout * l.cin * l.r * l.s)
            elif l.kind == BN:
                out.append(2 * l.cin)
            elif l.kind == FC:
                out.append(l.cout * l.cin + l.cout)
            elif l.kind == BIAS:
                out.append(l.cin)
            else:
                out.append(0)
        return out


def _conv_bn(net: NetSpec, src: int, cin: int, cout: int, r: int, stride: int, pad: int,
             relu: bool) -> int:
    c = net.add(Layer(CONV, in0=src, cin=cin, cout=cout, r=r, s=r, stride=stride, pad=pad))
    b = net.add(Layer(BN, in0=c, cin=cout, cout=cout))
    if relu:
        return net.add(Layer(RELU, in0=b, cin=cout, cout=cout))
    return b


def _bottleneck(net: NetSpec, src: int, cin: int, planes: int, stride: int,
                project: bool, variant: str, expansion: int = 4) -> int:
    cout = planes * expansion
    s1, s3 = (stride, 1) if variant == "v1" else (1, stride)
    shortcut = src
    if project:
        shortcut = _conv_bn(net, src, cin, cout, 1, stride, 0, relu=False)
    a = _conv_bn(net, src, cin, planes, 1, s1, 0, relu=True)
    b = _conv_bn(net, a, planes, planes, 3, s3, 1, relu=True)
    c = _conv_bn(net, b, planes, cout, 1, 1, 0, relu=False)
    d = net.add(Layer(ADD, in0=c, in1=shortcut, cin=cout, cout=cout))
    return net.add(Layer(RELU, in0=d, cin=cout, cout=cout))


def _basic_block(net: NetSpec, src: int, cin: int, planes: int, stride: int, project: bool) -> int:
    """Two 3x3 convolutions (the first carries the stride), identity or 1x1 projection shortcut."""
    shortcut = src
    if project:
        shortcut = _conv_bn(net, src, cin, planes, 1, stride, 0, relu=False)
    a = _conv_bn(net, src, cin, planes, 3, stride, 1, relu=True)
    b = _conv_bn(net, a, planes, planes, 3, 1, 1, relu=False)
    d = net.add(Layer(ADD, in0=b, in1=shortcut, cin=planes, cout=planes))
    return net.add(Layer(RELU, in0=d, cin=planes, cout=planes))


def _head(net: NetSpec, src: int, cin: int, classes: int) -> None:
    g = net.add(Layer(GAP, in0=src, cin=cin, cout=cin))
    f = net.add(Layer(FC, in0=g, cin=cin, cout=classes))
    net.add(Layer(SOFTMAX_CE, in0=f, cin=classes, cout=1))


def bottleneck_unit(cin: int = 64, planes: int = 16, hw: int = 16, classes: int = 10) -> NetSpec:
    """One identity-shortcut bottleneck block followed by global average pooling,
    a fully connected layer and softmax cross-entropy (BASELINE configs[0])."""
    net = NetSpec(f"bottleneck_{cin}_{planes}_{hw}", cin, hw, hw, classes)
    out = _bottleneck(net, -1, cin, planes, 1, project=False, variant="v1",
                      expansion=cin // planes)
    _head(net, out, cin, classes)
    return net


def resnet(blocks=(3, 4, 6, 3), in_c: int = 3, in_hw: int = 224, classes: int = 1000,
           width: int = 64, variant: str = "v1", name: str = "", block: str = "bottleneck") -> NetSpec:
    """ImageNet-style ResNet: 7x7/2 stem, 3x3/2 max-pool, four stages of blocks, global
    average pooling, FC, softmax cross-entropy.  block "bottleneck": 1x1-3x3-1x1 blocks with
    four times wider output, projection shortcut on the first block of every stage; variant
    "v1" puts the stride of a down-sampling block on its first 1x1 convolution, "v1.5" on the
    3x3.  block "basic" (the 18- and 34-layer networks): two 3x3 convolutions per block,
    projection shortcut only where the shape changes."""
    assert variant in ("v1", "v1.5") and block in ("bottleneck", "basic")
    net = NetSpec(name or f"resnet_{'-'.join(map(str, blocks))}_w{width}", in_c, in_hw, in_hw, classes)
    x = _conv_bn(net, -1, in_c, width, 7, 2, 3, relu=True)
    x = net.add(Layer(MAXPOOL, in0=x, cin=width, cout=width, r=3, s=3, stride=2, pad=1))
    cin = width
    for stage, nblk in enumerate(blocks):
        planes = width << stage
        for b in range(nblk):
            stride = 2 if (stage > 0 and b == 0) else 1
            if block == "basic":
                x = _basic_block(net, x, cin, planes, stride, project=(stride != 1 or cin != planes))
                cin = planes
            else:
                x = _bottleneck(net, x, cin, planes, stride, project=(b == 0), variant=variant)
                cin = planes * 4
    _head(net, x, cin, classes)
    return net


def vgg(cfg=((64, 64), (128, 128), (256, 256, 256), (512, 512, 512), (512, 512, 512)), in_c: int = 3,
        in_hw: int = 224, classes: int = 1000, fc: int = 4096, name: str = "") -> NetSpec:
    """VGG-style network: stages of 3x3 convolutions (padding 1) with a per-channel bias and
    ReLU, a 2x2 / 2 max-pool after every stage, then FC-ReLU-FC-ReLU-FC over the flattened map
    and softmax cross-entropy.  The default is configuration D of Simonyan & Zisserman (16
    weight layers).  Dropout is not part of the step here."""
    net = NetSpec(name or f"vgg_{sum(len(st) for st in cfg) + 3}", in_c, in_hw, in_hw, classes)
    x, c, hw = -1, in_c, in_hw
    for stage in cfg:
        for cout in stage:
            x = net.add(Layer(CONV, in0=x, cin=c, cout=cout, r=3, s=3, stride=1, pad=1))
            x = net.add(Layer(BIAS, in0=x, cin=cout, cout=cout))
            x = net.add(Layer(RELU, in0=x, cin=cout, cout=cout))
            c = cout
        x = net.add(Layer(MAXPOOL, in0=x, cin=c, cout=c, r=2, s=2, stride=2, pad=0))
        hw //= 2
    feat = c * hw * hw
    for width in (fc, fc):
        x = net.add(Layer(FC, in0=x, cin=feat, cout=width))
        x = net.add(Layer(RELU, in0=x, cin=width, cout=width))
        feat = width
    x = net.add(Layer(FC, in0=x, cin=feat, cout=classes))
    net.add(Layer(SOFTMAX_CE, in0=x, cin=classes, cout=1))
    return net


def vgg16(**kw) -> NetSpec:
    return vgg(name="vgg16", **kw)


def resnet18(**kw) -> NetSpec:
    return resnet((2, 2, 2, 2), name="resnet18", block="basic", **kw)


def resnet34(**kw) -> NetSpec:
    return resnet((3, 4, 6, 3), name="resnet34", block="basic", **kw)


def resnet50(**kw) -> NetSpec:
    return resnet((3, 4, 6, 3), name="resnet50", **kw)


def resnet101(**kw) -> NetSpec:
    return resnet((3, 4, 23, 3), name="resnet101", **kw)


def resnet152(**kw) -> NetSpec:
    return resnet((3, 8, 36, 3), name="resnet152", **kw)


def param_count(net: NetSpec) -> int:
    return int(sum(net.param_sizes()))


def _layer_seed(seed: int, layer_id: int) -> int:
    return int(splitmix64(seed, layer_id, 1)[0])


def init_params(net: NetSpec, seed: int = 42) -> List[np.ndarray]:
    """One float32 array per layer (empty for parameter-free layers).
    conv: OIHW weights ~ N(0, 2/fan_in), fan_in = cin*r*s.
    bias: C zeros.
    bn:   [gamma (C ones) | beta (C zeros)].
    fc:   [W (cout x cin, row major) ~ N(0, 2/cin) | b (cout zeros)].
    Layer i draws from its own stream, seeded by output i of splitmix64(seed)."""
    out = []
    for i, l in enumerate(net.layers):
        if l.kind == CONV:
            n = l.cout * l.cin * l.r * l.s
            std = np.sqrt(2.0 / (l.cin * l.r * l.s))
            out.append((normal(_layer_seed(seed, i), n) * std).astype(np.float32))
        elif l.kind == BN:
            out.append(np.concatenate([np.ones(l.cin, np.float32), np.zeros(l.cin, np.float32)]))
        elif l.kind == FC:
            n = l.cout * l.cin
            std = np.sqrt(2.0 / l.cin)
            w = (normal(_layer_seed(seed, i), n) * std).astype(np.float32)
            out.append(np.concatenate([w, np.zeros(l.cout, np.float32)]))
        elif l.kind == BIAS:
            out.append(np.zeros(l.cin, np.float32))
        else:
            out.append(np.zeros(0, np.float32))
    return out


def make_batch(net: NetSpec, k: int, step: int = 0):
    """(images float32 [k, C, H, W] ~ N(0,1) from seed 1000+step,
        labels int32 [k] uniform in [0, classes) from seed 2000+step)."""
    n = k * net.in_c * net.in_h * net.in_w
    img = normal(1000 + step, n).astype(np.float32).reshape(k, net.in_c, net.in_h, net.in_w)
    lab = labels_uniform(2000 + step, k, net.classes)
    return img, lab
