"""Layer-shape enumerators for the five benchmark workloads.

A "layer" here is one preconditioned layer of a network: it owns one
Kronecker-factor pair (A from the layer's input activations, G from the
gradients w.r.t. its outputs; paper Sec. II-B).  Only shapes are described.

The ResNet enumerators follow the bottleneck architecture with the stride on
the 3x3 convolution; with ``has_bias=0`` on convolutions their packed-triangle
totals reproduce the paper's Table II (#As / #Gs) and the extreme sizes quoted
in Sec. IV-A, which the CPU tests assert.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List

LINEAR = 0
CONV2D = 1


@dataclass(frozen=True)
class Layer:
    kind: int          # LINEAR or CONV2D
    n: int = 0         # conv: batch size
    c_in: int = 0
    h: int = 0         # conv: input height
    w: int = 0         # conv: input width
    c_out: int = 0
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0       # zero padding of the height (and of the width unless pad_w is given)
    pad_w: int = -1    # zero padding of the width; -1 = same as pad
    rows: int = 0      # linear: number of rows (batch, or batch*seq)
    has_bias: int = 1  # 1 -> a ones column is appended last to the activations
    name: str = ""

    @property
    def ph(self) -> int:
        return self.pad

    @property
    def pw(self) -> int:
        return self.pad if self.pad_w < 0 else self.pad_w

    @property
    def oh(self) -> int:
        return (self.h + 2 * self.ph - self.kh) // self.stride + 1

    @property
    def ow(self) -> int:
        return (self.w + 2 * self.pw - self.kw) // self.stride + 1

    @property
    def R(self) -> int:
        """Rows of the (im2col'd) activation matrix = samples the factor averages over."""
        return self.rows if self.kind == LINEAR else self.n * self.oh * self.ow

    @property
    def dA(self) -> int:
        return self.c_in * self.kh * self.kw + self.has_bias

    @property
    def dG(self) -> int:
        return self.c_out

    @property
    def act_shape(self):
        return (self.rows, self.c_in) if self.kind == LINEAR else (self.n, self.c_in, self.h, self.w)

    @property
    def gout_shape(self):
        return (self.rows, self.c_out) if self.kind == LINEAR else (self.n, self.c_out, self.oh, self.ow)


def linear(rows, c_in, c_out, has_bias=1, name="") -> Layer:
    return Layer(kind=LINEAR, rows=rows, c_in=c_in, c_out=c_out, has_bias=has_bias, name=name)


def conv(n, c_in, h, w, c_out, k, stride=1, pad=0, has_bias=1, name="") -> Layer:
    return Layer(kind=CONV2D, n=n, c_in=c_in, h=h, w=w, c_out=c_out, kh=k, kw=k,
                 stride=stride, pad=pad, has_bias=has_bias, name=name)


def fc_layers() -> List[Layer]:
    return [linear(32, 64, 32, name="fc")]


def cnn_layers(batch=32) -> List[Layer]:
    chans = [3, 32, 64, 128, 128]
    ls = [conv(batch, chans[i], 32, 32, chans[i + 1], 3, 1, 1, name=f"conv{i + 1}") for i in range(4)]
    ls.append(linear(batch, 128, 10, name="fc"))
    return ls


def resnet_layers(blocks, batch=32, image=224, classes=1000, conv_bias=1) -> List[Layer]:
    """Bottleneck ResNet (stride on the 3x3), widths 64/128/256/512, expansion 4."""
    ls = [conv(batch, 3, image, image, 64, 7, 2, 3, conv_bias, name="stem")]
    res = (image + 2 * 3 - 7) // 2 + 1          # stem output
    res = (res + 2 * 1 - 3) // 2 + 1            # 3x3/2 max-pool, pad 1
    c_prev = 64
    for s, (nb, width) in enumerate(zip(blocks, (64, 128, 256, 512))):
        for b in range(nb):
            stride = 2 if (s > 0 and b == 0) else 1
            tag = f"s{s + 1}b{b}"
            ls.append(conv(batch, c_prev, res, res, width, 1, 1, 0, conv_bias, name=tag + ".conv1"))
            ls.append(conv(batch, width, res, res, width, 3, stride, 1, conv_bias, name=tag + ".conv2"))
            res_out = (res + 2 - 3) // stride + 1
            ls.append(conv(batch, width, res_out, res_out, 4 * width, 1, 1, 0, conv_bias, name=tag + ".conv3"))
            if b == 0:
                ls.append(conv(batch, c_prev, res, res, 4 * width, 1, stride, 0, conv_bias, name=tag + ".proj"))
            res = res_out
            c_prev = 4 * width
    ls.append(linear(batch, c_prev, classes, 1, name="fc"))
    return ls


def densenet_layers(blocks=(6, 12, 48, 32), growth=32, bn_size=4, batch=16, image=224, classes=1000,
                    conv_bias=1) -> List[Layer]:
    """DenseNet (DenseNet-201 by default): 7x7/2 stem to 2*growth channels, 3x3/2 max-pool, dense
    blocks whose layers are a 1x1 bottleneck to bn_size*growth channels followed by a 3x3 to `growth`
    channels (input = concatenation of everything before), halving 1x1 transitions with 2x2 average
    pooling between blocks, linear classifier."""
    ls = [conv(batch, 3, image, image, 2 * growth, 7, 2, 3, conv_bias, name="stem")]
    res = (image + 2 * 3 - 7) // 2 + 1
    res = (res + 2 * 1 - 3) // 2 + 1
    c = 2 * growth
    for b, nl in enumerate(blocks):
        for i in range(nl):
            ls.append(conv(batch, c, res, res, bn_size * growth, 1, 1, 0, conv_bias, name=f"d{b + 1}l{i}.conv1"))
            ls.append(conv(batch, bn_size * growth, res, res, growth, 3, 1, 1, conv_bias, name=f"d{b + 1}l{i}.conv2"))
            c += growth
        if b + 1 < len(blocks):
            ls.append(conv(batch, c, res, res, c // 2, 1, 1, 0, conv_bias, name=f"t{b + 1}"))
            c //= 2
            res //= 2
    ls.append(linear(batch, c, classes, 1, name="fc"))
    return ls


def inception_v4_layers(batch=16, image=224, classes=1000, conv_bias=1) -> List[Layer]:
    """Inception-v4: stem (unpadded 3x3 convolutions, one padded; a 1x7 / 7x1 pair), 4 x Inception-A,
    Reduction-A, 7 x Inception-B, Reduction-B, 3 x Inception-C, linear classifier.  Windows such as
    1x7 are padded along their long side only; pooling branches contribute no preconditioned layer
    except their 1x1 projections."""
    ls: List[Layer] = []
    sz = lambda r, k, s, p: (r + 2 * p - k) // s + 1

    def add(name, cin, res, cout, kh, kw, stride=1, ph=0, pw=0):
        ls.append(Layer(kind=CONV2D, n=batch, c_in=cin, h=res, w=res, c_out=cout, kh=kh, kw=kw, stride=stride,
                        pad=ph, pad_w=pw, has_bias=conv_bias, name=name))

    r = image
    add("stem.c1", 3, r, 32, 3, 3, 2); r = sz(r, 3, 2, 0)
    add("stem.c2", 32, r, 32, 3, 3); r = sz(r, 3, 1, 0)
    add("stem.c3", 32, r, 64, 3, 3, 1, 1, 1)
    add("stem.3a", 64, r, 96, 3, 3, 2); r = sz(r, 3, 2, 0)            # beside a 3x3/2 max-pool: 64 + 96 = 160
    add("stem.4a.b0c1", 160, r, 64, 1, 1)
    add("stem.4a.b0c2", 64, r, 96, 3, 3)
    add("stem.4a.b1c1", 160, r, 64, 1, 1)
    add("stem.4a.b1c2", 64, r, 64, 1, 7, 1, 0, 3)
    add("stem.4a.b1c3", 64, r, 64, 7, 1, 1, 3, 0)
    add("stem.4a.b1c4", 64, r, 96, 3, 3); r = sz(r, 3, 1, 0)          # 96 + 96 = 192
    add("stem.5a", 192, r, 192, 3, 3, 2); r = sz(r, 3, 2, 0)          # beside a max-pool: 384
    for b in range(4):
        t = f"A{b}."
        add(t + "b0", 384, r, 96, 1, 1)
        add(t + "b1c1", 384, r, 64, 1, 1); add(t + "b1c2", 64, r, 96, 3, 3, 1, 1, 1)
        add(t + "b2c1", 384, r, 64, 1, 1); add(t + "b2c2", 64, r, 96, 3, 3, 1, 1, 1); add(t + "b2c3", 96, r, 96, 3, 3, 1, 1, 1)
        add(t + "b3", 384, r, 96, 1, 1)
    add("RA.b0", 384, r, 384, 3, 3, 2)
    add("RA.b1c1", 384, r, 192, 1, 1); add("RA.b1c2", 192, r, 224, 3, 3, 1, 1, 1); add("RA.b1c3", 224, r, 256, 3, 3, 2)
    r = sz(r, 3, 2, 0)                                                  # 384 + 256 + 384 (pool) = 1024
    for b in range(7):
        t = f"B{b}."
        add(t + "b0", 1024, r, 384, 1, 1)
        add(t + "b1c1", 1024, r, 192, 1, 1); add(t + "b1c2", 192, r, 224, 1, 7, 1, 0, 3); add(t + "b1c3", 224, r, 256, 7, 1, 1, 3, 0)
        add(t + "b2c1", 1024, r, 192, 1, 1); add(t + "b2c2", 192, r, 192, 7, 1, 1, 3, 0); add(t + "b2c3", 192, r, 224, 1, 7, 1, 0, 3)
        add(t + "b2c4", 224, r, 224, 7, 1, 1, 3, 0); add(t + "b2c5", 224, r, 256, 1, 7, 1, 0, 3)
        add(t + "b3", 1024, r, 128, 1, 1)
    add("RB.b0c1", 1024, r, 192, 1, 1); add("RB.b0c2", 192, r, 192, 3, 3, 2)
    add("RB.b1c1", 1024, r, 256, 1, 1); add("RB.b1c2", 256, r, 256, 1, 7, 1, 0, 3); add("RB.b1c3", 256, r, 320, 7, 1, 1, 3, 0)
    add("RB.b1c4", 320, r, 320, 3, 3, 2)
    r = sz(r, 3, 2, 0)                                                  # 192 + 320 + 1024 (pool) = 1536
    for b in range(3):
        t = f"C{b}."
        add(t + "b0", 1536, r, 256, 1, 1)
        add(t + "b1c1", 1536, r, 384, 1, 1); add(t + "b1c2a", 384, r, 256, 1, 3, 1, 0, 1); add(t + "b1c2b", 384, r, 256, 3, 1, 1, 1, 0)
        add(t + "b2c1", 1536, r, 384, 1, 1); add(t + "b2c2", 384, r, 448, 3, 1, 1, 1, 0); add(t + "b2c3", 448, r, 512, 1, 3, 1, 0, 1)
        add(t + "b2c4a", 512, r, 256, 1, 3, 1, 0, 1); add(t + "b2c4b", 512, r, 256, 3, 1, 1, 1, 0)
        add(t + "b3", 1536, r, 256, 1, 1)
    ls.append(linear(batch, 1536, classes, 1, name="fc"))
    return ls


def bert_large_layers(blocks=24, hidden=1024, ffn=4096, tokens=32 * 128) -> List[Layer]:
    ls = []
    for b in range(blocks):
        for nm in ("q", "k", "v", "o"):
            ls.append(linear(tokens, hidden, hidden, name=f"b{b}.{nm}"))
        ls.append(linear(tokens, hidden, ffn, name=f"b{b}.ffn1"))
        ls.append(linear(tokens, ffn, hidden, name=f"b{b}.ffn2"))
    return ls


# name -> (config id used in seeding, hyper-parameters)
CONFIGS = {
    "fc":    dict(cid=1, xi=0.95, gamma=0.03, relu=True),
    "cnn":   dict(cid=2, xi=0.95, gamma=0.03, relu=True),
    "r50":   dict(cid=3, xi=0.95, gamma=0.03, relu=True),
    "r152":  dict(cid=4, xi=0.95, gamma=0.03, relu=True),
    "bertl": dict(cid=5, xi=0.95, gamma=0.01, relu=False),
    "d201":  dict(cid=6, xi=0.95, gamma=0.03, relu=True),
    "iv4":   dict(cid=7, xi=0.95, gamma=0.03, relu=True),
}


def config_layers(name: str, batch: int | None = None) -> List[Layer]:
    if name == "fc":
        return fc_layers()
    if name == "cnn":
        return cnn_layers(batch or 32)
    if name == "r50":
        return resnet_layers((3, 4, 6, 3), batch or 32)
    if name == "r152":
        return resnet_layers((3, 8, 36, 3), batch or 32)
    if name == "bertl":
        return bert_large_layers()
    if name == "d201":
        return densenet_layers(batch=batch or 16)
    if name == "iv4":
        return inception_v4_layers(batch=batch or 16)
    raise KeyError(name)


def config_hparams(name: str) -> dict:
    return dict(CONFIGS[name])


def shrink(layers: List[Layer], batch: int) -> List[Layer]:
    """Same layer set at a smaller batch (conv) / row count (linear); used by tests."""
    out = []
    for l in layers:
        out.append(replace(l, n=batch) if l.kind == CONV2D else replace(l, rows=min(l.rows, batch)))
    return out


def flops(layers: List[Layer]) -> dict:
    """Algorithmic work per step: factors count one triangle (R*d*(d+1) flops per factor),
    the inverse d^3 per matrix, preconditioning the two dense products."""
    fa = sum(l.R * l.dA * (l.dA + 1) for l in layers)
    fg = sum(l.R * l.dG * (l.dG + 1) for l in layers)
    inv = sum(l.dA ** 3 + l.dG ** 3 for l in layers)
    pre = sum(2 * l.dG * l.dG * l.dA + 2 * l.dG * l.dA * l.dA for l in layers)
    return dict(factor_a=fa, factor_g=fg, inverse=inv, precondition=pre,
                total=fa + fg + inv + pre)
