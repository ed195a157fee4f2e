"""Layer shape descriptions (no arithmetic of the method lives here)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

DENSE, CONV, GN = "dense", "conv", "gn"


@dataclass(frozen=True)
class Layer:
    """One parameterised layer whose per-example weight gradient is privatised.

    dense : x [T, cin], dy [T, cout]           (h = T tokens, w = 1)
    conv  : x [cin, h, w], dy [cout, oh, ow]   (cross-correlation, zero padding)
    gn    : x [c, h, w] (pre-normalisation input), dy [c, h, w]; cin == cout == c
    """
    kind: str
    cin: int
    cout: int
    h: int = 1
    w: int = 1
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0
    has_bias: bool = False
    gn_groups: int = 0
    gn_eps: float = 1e-5
    name: str = ""

    @property
    def oh(self) -> int:
        if self.kind == CONV:
            return (self.h + 2 * self.pad - self.kh) // self.stride + 1
        return self.h

    @property
    def ow(self) -> int:
        if self.kind == CONV:
            return (self.w + 2 * self.pad - self.kw) // self.stride + 1
        return self.w

    @property
    def x_shape(self):
        if self.kind == DENSE:
            return (self.h, self.cin)
        return (self.cin, self.h, self.w)

    @property
    def dy_shape(self):
        if self.kind == DENSE:
            return (self.h, self.cout)
        if self.kind == GN:
            return (self.cin, self.h, self.w)
        return (self.cout, self.oh, self.ow)

    @property
    def pw(self) -> int:
        """Number of weight (or GroupNorm scale) parameters."""
        if self.kind == GN:
            return self.cin
        return self.cout * self.cin * self.kh * self.kw

    @property
    def pb(self) -> int:
        """Number of bias (or GroupNorm shift) parameters."""
        if self.kind == GN:
            return self.cin
        return self.cout if self.has_bias else 0

    @property
    def w_shape(self):
        if self.kind == GN:
            return (self.cin,)
        if self.kind == DENSE:
            return (self.cout, self.cin)
        return (self.cout, self.cin, self.kh, self.kw)

    @property
    def flops(self) -> int:
        """Multiply-adds x2 of one example's weight-gradient contraction."""
        if self.kind == GN:
            return 3 * self.cin * self.h * self.w
        s = self.oh * self.ow
        return 2 * self.cout * self.cin * self.kh * self.kw * s

    def in_bytes(self, elem_bytes: int) -> int:
        """Bytes of x and dy of one example."""
        nx = 1
        for d in self.x_shape:
            nx *= d
        ny = 1
        for d in self.dy_shape:
            ny *= d
        return (nx + ny) * elem_bytes


def conv(cin, cout, k, stride, hw, bias=False, name="") -> Layer:
    return Layer(CONV, cin, cout, hw, hw, k, k, stride, (k - 1) // 2, bias, name=name)


def dense(cin, cout, tokens=1, bias=True, name="") -> Layer:
    return Layer(DENSE, cin, cout, tokens, 1, has_bias=bias, name=name)


def gn_affine(c, hw, groups, name="") -> Layer:
    return Layer(GN, c, c, hw, hw, gn_groups=groups, name=name)


def tiny_mlp_layers() -> List[Layer]:
    return [dense(784, 256, name="fc1"), dense(256, 10, name="fc2")]


def resnet20_layers(with_gn: bool = True, hw: int = 32) -> List[Layer]:
    """CIFAR ResNet-20: 19 3x3 convs (no bias, parameter-free shortcuts), a GroupNorm(8)
    affine after every conv, and a 64->10 dense layer with bias."""
    out: List[Layer] = []

    def add(cin, cout, stride, res, tag):
        c = conv(cin, cout, 3, stride, res, name=f"conv{tag}")
        out.append(c)
        if with_gn:
            out.append(gn_affine(cout, c.oh, 8, name=f"gn{tag}"))
        return c.oh

    res = add(3, 16, 1, hw, "0")
    widths = [16, 32, 64]
    cin = 16
    idx = 1
    for si, wd in enumerate(widths):
        for b in range(6):
            stride = 2 if (si > 0 and b == 0) else 1
            res = add(cin, wd, stride, res, str(idx))
            cin = wd
            idx += 1
    out.append(dense(64, 10, name="fc"))
    return out


def resnet_bottleneck_layers(blocks=(3, 4, 6, 3), hw: int = 224, num_classes: int = 1000,
                             gn_groups: int = 0) -> List[Layer]:
    """Bottleneck ResNet (50: blocks 3,4,6,3; 101: 3,4,23,3) with the stride on the 3x3 conv of each
    stage's first bottleneck: bias-free convs plus one dense layer with bias.  With gn_groups > 0 every
    conv is followed by a GroupNorm whose scale/shift gradients are part of the set (its input is the
    conv's output).  `hw` scales the input resolution (224 is the real one)."""
    out: List[Layer] = []

    def add(layer: Layer):
        out.append(layer)
        if gn_groups:
            out.append(gn_affine(layer.cout, layer.oh, gn_groups, name=layer.name + ".gn"))
        return layer

    c1 = add(conv(3, 64, 7, 2, hw, name="conv1"))
    res = (c1.oh + 2 - 3) // 2 + 1          # 3x3 stride-2 max-pool, pad 1
    cin = 64
    for si, (width, nb) in enumerate(zip((64, 128, 256, 512), blocks)):
        cout = 4 * width
        for b in range(nb):
            stride = 2 if (si > 0 and b == 0) else 1
            tag = f"s{si + 1}b{b + 1}"
            add(conv(cin, width, 1, 1, res, name=tag + ".c1"))
            c2 = add(conv(width, width, 3, stride, res, name=tag + ".c2"))
            add(conv(width, cout, 1, 1, c2.oh, name=tag + ".c3"))
            if b == 0:
                add(conv(cin, cout, 1, stride, res, name=tag + ".down"))
            res = c2.oh
            cin = cout
    out.append(dense(2048, num_classes, name="fc"))
    return out


def resnet50_layers(hw: int = 224, num_classes: int = 1000) -> List[Layer]:
    """ResNet-50: 53 bias-free convs plus one dense layer with bias (no GroupNorm gradients)."""
    return resnet_bottleneck_layers((3, 4, 6, 3), hw, num_classes, 0)


def resnet18_layers(hw: int = 32, num_classes: int = 10, gn_groups: int = 32) -> List[Layer]:
    """CIFAR-style ResNet-18 with GroupNorm: a 3x3 stem, four stages of two basic blocks (two 3x3
    convs each), 1x1 stride-2 projection shortcuts at the start of stages 2-4, a GroupNorm affine
    after every conv, dense 512 -> classes with bias."""
    out: List[Layer] = []

    def add(layer: Layer):
        out.append(layer)
        if gn_groups:
            out.append(gn_affine(layer.cout, layer.oh, gn_groups, name=layer.name + ".gn"))
        return layer

    res = add(conv(3, 64, 3, 1, hw, name="conv1")).oh
    cin = 64
    for si, width in enumerate((64, 128, 256, 512)):
        for b in range(2):
            stride = 2 if (si > 0 and b == 0) else 1
            tag = f"s{si + 1}b{b + 1}"
            c1 = add(conv(cin, width, 3, stride, res, name=tag + ".c1"))
            add(conv(width, width, 3, 1, c1.oh, name=tag + ".c2"))
            if stride == 2:
                add(conv(cin, width, 1, 2, res, name=tag + ".down"))
            res = c1.oh
            cin = width
    out.append(dense(512, num_classes, name="fc"))
    return out
