"""Layer tables of the CNN architectures named by the benchmark configurations.

A network is a list of `Layer` records.  Layer `l` reads the output of layer
`in_from` (-1 = the network input) and, when `res_from >= 0`, adds the output of
layer `res_from` before its activation.  Convolution weights are OIHW
(`[c_out][c_in/groups][k][k]`), FC weights `[c_out][c_in]` where the FC input is
the producing tensor flattened in (channel, row, column) order.

Only shapes live here; there is no arithmetic of the method in this module.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

OP_CONV, OP_MAXPOOL, OP_GAVGPOOL, OP_FC = 0, 1, 2, 3
ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2


@dataclass(frozen=True)
class Layer:
    op: int
    c_in: int
    c_out: int
    k: int = 1
    stride: int = 1
    pad: int = 0
    groups: int = 1
    act: int = ACT_NONE
    in_from: int = -1
    res_from: int = -1
    has_bn: bool = False  # weight generator folds a seeded BN into this conv
    name: str = ""


class _Builder:
    def __init__(self) -> None:
        self.layers: List[Layer] = []

    @property
    def last(self) -> int:
        return len(self.layers) - 1

    def add(self, **kw) -> int:
        kw.setdefault("in_from", self.last)
        self.layers.append(Layer(**kw))
        return self.last

    def conv(self, cin, cout, k, s, p, act, *, groups=1, in_from=None, res_from=-1, bn=True, name=""):
        kw = dict(op=OP_CONV, c_in=cin, c_out=cout, k=k, stride=s, pad=p, groups=groups, act=act,
                  res_from=res_from, has_bn=bn, name=name)
        if in_from is not None:
            kw["in_from"] = in_from
        return self.add(**kw)

    def maxpool(self, c, k, s, p, name=""):
        return self.add(op=OP_MAXPOOL, c_in=c, c_out=c, k=k, stride=s, pad=p, name=name)

    def gavgpool(self, c, name="gap"):
        return self.add(op=OP_GAVGPOOL, c_in=c, c_out=c, name=name)

    def fc(self, cin, cout, act=ACT_NONE, name=""):
        return self.add(op=OP_FC, c_in=cin, c_out=cout, act=act, name=name)


def tiny() -> Tuple[List[Layer], Tuple[int, int, int]]:
    b = _Builder()
    b.conv(3, 16, 3, 1, 1, ACT_RELU, bn=False, name="c1")
    b.conv(16, 32, 3, 1, 1, ACT_RELU, bn=False, name="c2")
    b.maxpool(32, 2, 2, 0, name="p1")
    b.conv(32, 32, 3, 1, 1, ACT_RELU, bn=False, name="c3")
    b.conv(32, 64, 3, 1, 1, ACT_RELU, bn=False, name="c4")
    b.maxpool(64, 2, 2, 0, name="p2")
    b.fc(64 * 8 * 8, 10, name="fc")
    return b.layers, (3, 32, 32)


def _resnet(block: str, counts, num_classes=1000):
    b = _Builder()
    b.conv(3, 64, 7, 2, 3, ACT_RELU, name="stem")
    b.maxpool(64, 3, 2, 1, name="stem.pool")
    cin = 64
    for li, (n, width) in enumerate(zip(counts, (64, 128, 256, 512))):
        for bi in range(n):
            s = 2 if (li > 0 and bi == 0) else 1
            x = b.last
            nm = f"l{li + 1}b{bi}"
            if block == "basic":
                cout = width
                skip = x
                if s != 1 or cin != cout:
                    skip = b.conv(cin, cout, 1, s, 0, ACT_NONE, in_from=x, name=nm + ".ds")
                b.conv(cin, width, 3, s, 1, ACT_RELU, in_from=x, name=nm + ".c1")
                b.conv(width, cout, 3, 1, 1, ACT_RELU, res_from=skip, name=nm + ".c2")
            else:
                cout = 4 * width
                skip = x
                if s != 1 or cin != cout:
                    skip = b.conv(cin, cout, 1, s, 0, ACT_NONE, in_from=x, name=nm + ".ds")
                b.conv(cin, width, 1, 1, 0, ACT_RELU, in_from=x, name=nm + ".c1")
                b.conv(width, width, 3, s, 1, ACT_RELU, name=nm + ".c2")
                b.conv(width, cout, 1, 1, 0, ACT_RELU, res_from=skip, name=nm + ".c3")
            cin = cout
    b.gavgpool(cin)
    b.fc(cin, num_classes, name="fc")
    return b.layers, (3, 224, 224)


def resnet18():
    return _resnet("basic", (2, 2, 2, 2))


def resnet50():
    return _resnet("bottleneck", (3, 4, 6, 3))


def vgg16():
    b = _Builder()
    cin = 3
    i = 0
    for v in (64, 64, "M", 128, 128, "M", 256, 256, 256, "M", 512, 512, 512, "M", 512, 512, 512, "M"):
        if v == "M":
            b.maxpool(cin, 2, 2, 0, name=f"pool{i}")
        else:
            i += 1
            b.conv(cin, v, 3, 1, 1, ACT_RELU, bn=False, name=f"c{i}")
            cin = v
    b.fc(512 * 7 * 7, 4096, ACT_RELU, name="fc1")
    b.fc(4096, 4096, ACT_RELU, name="fc2")
    b.fc(4096, 1000, name="fc3")
    return b.layers, (3, 224, 224)


def mobilenet_v2():
    b = _Builder()
    b.conv(3, 32, 3, 2, 1, ACT_RELU6, name="stem")
    cin = 32
    bi = 0
    for t, c, n, s in ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
                       (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)):
        for r in range(n):
            stride = s if r == 0 else 1
            x = b.last
            hid = cin * t
            nm = f"ir{bi}"
            if t != 1:
                b.conv(cin, hid, 1, 1, 0, ACT_RELU6, in_from=x, name=nm + ".expand")
            b.conv(hid, hid, 3, stride, 1, ACT_RELU6, groups=hid, name=nm + ".dw")
            res = x if (stride == 1 and cin == c) else -1
            b.conv(hid, c, 1, 1, 0, ACT_NONE, res_from=res, name=nm + ".project")
            cin = c
            bi += 1
    b.conv(cin, 1280, 1, 1, 0, ACT_RELU6, name="head")
    b.gavgpool(1280)
    b.fc(1280, 1000, name="fc")
    return b.layers, (3, 224, 224)


NETS = {"tiny": tiny, "resnet18": resnet18, "resnet50": resnet50, "vgg16": vgg16,
        "mobilenet_v2": mobilenet_v2}


def build_net(name: str):
    """Return (layers, (C, H, W) input shape) of a named architecture."""
    return NETS[name]()


def layer_shapes(layers, in_shape):
    """Per-layer output shape (C, H, W), from the usual floor((H + 2p - k)/s) + 1 rule."""
    out = []
    for L in layers:
        c, h, w = in_shape if L.in_from < 0 else out[L.in_from]
        if L.op == OP_CONV or L.op == OP_MAXPOOL:
            assert c == L.c_in, (L, c)
            ho = (h + 2 * L.pad - L.k) // L.stride + 1
            wo = (w + 2 * L.pad - L.k) // L.stride + 1
            out.append((L.c_out, ho, wo))
        elif L.op == OP_GAVGPOOL:
            out.append((c, 1, 1))
        else:
            assert c * h * w == L.c_in, (L, c, h, w)
            out.append((L.c_out, 1, 1))
    return out


def net_macs(layers, in_shape):
    """Multiply-accumulates per layer (pools count zero)."""
    shp = layer_shapes(layers, in_shape)
    macs = []
    for L, (c, h, w) in zip(layers, shp):
        if L.op == OP_CONV:
            macs.append(h * w * L.c_out * (L.c_in // L.groups) * L.k * L.k)
        elif L.op == OP_FC:
            macs.append(L.c_in * L.c_out)
        else:
            macs.append(0)
    return macs


def net_params(layers):
    """Weights + one bias per output channel, over conv and FC layers."""
    n = 0
    for L in layers:
        if L.op == OP_CONV:
            n += L.c_out * (L.c_in // L.groups) * L.k * L.k + L.c_out
        elif L.op == OP_FC:
            n += L.c_out * L.c_in + L.c_out
    return n
