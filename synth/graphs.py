"""Tenant operator graphs (flat operator lists in execution order).

A tenant is a model M_n = [O_n,1 ... O_n,i] (Section 4.1): list order is
execution order, every operator reads tensors written earlier in the list.
Tensor shapes are logical (n, c, h, w); logical element order is NCHW for
activations and [out][in/groups][kh][kw] for weights.  Token tensors of the
transformer tenant use c = features, h = sequence position, w = 1; attention
score tensors use n = batch*heads, c = key position, h = query position.

Nothing here computes anything: builders emit shapes and parameter recipes,
``materialise`` draws the seeded numbers.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple
import math
import numpy as np

from .rng import splitmix64_uniform, splitmix64_normal, bf16_round

KINDS = ("conv", "dwconv", "gemm", "bgemm_qk", "bgemm_pv", "maxpool", "gavgpool",
         "affine", "add", "layernorm", "softmax", "act", "scale", "concat", "avgpool")
ACTS = ("none", "relu", "relu6", "gelu", "hswish", "hsigmoid")
BN_EPS = 1e-5
LN_EPS = 1e-12


@dataclass
class Op:
    kind: str
    in0: int
    out: int
    in1: int = -1
    res: int = -1
    w: int = -1          # indices into Tenant.params, -1 = absent
    bias: int = -1
    scale: int = -1
    shift: int = -1
    cin: int = 0
    cout: int = 0
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0
    groups: int = 1      # conv groups; attention: number of heads
    act: str = "none"
    alpha: float = 1.0   # attention score scale
    eps: float = 0.0     # layernorm epsilon


@dataclass
class Param:
    shape: Tuple[int, ...]
    init: str            # 'he_uniform' | 'zeros' | 'ones' | 'uniform'
    fan_in: int = 1
    fold: float = 1.0    # multiplicative BN fold factor applied in fp64


@dataclass
class Tenant:
    name: str
    dtype: str           # 'f32' | 'bf16'
    batch: int
    tensors: List[Tuple[int, int, int, int]] = field(default_factory=list)
    ops: List[Op] = field(default_factory=list)
    params: List[Param] = field(default_factory=list)
    input: int = 0
    output: int = 0
    input_dist: str = "uniform"   # 'uniform' U[-1,1) | 'normal002' N(0, 0.02^2)
    # channel windows: tensor index -> (index of the wider tensor it lives in, first channel).  A window shares the wider
    # tensor's storage, so writing windows one after the other concatenates along channels without a copy.
    views: Dict[int, Tuple[int, int]] = field(default_factory=dict)


class _B:
    """Small helper that appends tensors / params / ops to a Tenant."""

    def __init__(self, name, dtype, batch):
        self.t = Tenant(name, dtype, batch)

    def tensor(self, n, c, h, w):
        self.t.tensors.append((n, c, h, w))
        return len(self.t.tensors) - 1

    def param(self, shape, init, fan_in=1, fold=1.0):
        self.t.params.append(Param(tuple(shape), init, fan_in, fold))
        return len(self.t.params) - 1

    def shape(self, i):
        return self.t.tensors[i]

    def view(self, base, c_off, c):
        """Channels [c_off, c_off + c) of tensor ``base`` as a tensor of its own (shared storage)."""
        n, cb, h, w = self.shape(base)
        assert base not in self.t.views and 0 <= c_off and c_off + c <= cb
        y = self.tensor(n, c, h, w)
        self.t.views[y] = (base, c_off)
        return y

    def _out(self, out, shape):
        if out is None:
            return self.tensor(*shape)
        assert self.shape(out) == tuple(shape)
        return out

    def conv(self, x, cout, k, stride=1, pad=0, act="none", res=-1, bn=False, groups=1, out=None):
        n, c, h, w = self.shape(x)
        ho = (h + 2 * pad - k) // stride + 1
        wo = (w + 2 * pad - k) // stride + 1
        y = self._out(out, (n, cout, ho, wo))
        fan_in = (c // groups) * k * k
        fold = 1.0 / math.sqrt(1.0 + BN_EPS) if bn else 1.0
        wi = self.param((cout, c // groups, k, k), "he_uniform", fan_in, fold)
        bi = self.param((cout,), "zeros")
        kind = "dwconv" if (groups == c and groups == cout and groups > 1) else "conv"
        self.t.ops.append(Op(kind, x, y, res=res, w=wi, bias=bi, cin=c, cout=cout, kh=k, kw=k,
                             stride=stride, pad=pad, groups=groups, act=act))
        return y

    def gemm(self, x, cout, act="none", res=-1, flatten=False, fold=1.0):
        n, c, h, w = self.shape(x)
        if flatten:
            cin = c * h * w
            y = self.tensor(n, cout, 1, 1)
        else:
            cin = c
            y = self.tensor(n, cout, h, w)
        wi = self.param((cout, cin), "he_uniform", cin, fold)
        bi = self.param((cout,), "zeros")
        self.t.ops.append(Op("gemm", x, y, res=res, w=wi, bias=bi, cin=cin, cout=cout, act=act))
        return y

    def maxpool(self, x, k, stride, pad, out=None):
        n, c, h, w = self.shape(x)
        ho = (h + 2 * pad - k) // stride + 1
        wo = (w + 2 * pad - k) // stride + 1
        y = self._out(out, (n, c, ho, wo))
        self.t.ops.append(Op("maxpool", x, y, cin=c, cout=c, kh=k, kw=k, stride=stride, pad=pad))
        return y

    def gavgpool(self, x):
        n, c, h, w = self.shape(x)
        y = self.tensor(n, c, 1, 1)
        self.t.ops.append(Op("gavgpool", x, y, cin=c, cout=c))
        return y

    def affine(self, x, act="none", res=-1, init="uniform"):
        n, c, h, w = self.shape(x)
        y = self.tensor(n, c, h, w)
        sc = self.param((c,), init)
        sh = self.param((c,), init)
        self.t.ops.append(Op("affine", x, y, res=res, scale=sc, shift=sh, cin=c, cout=c, act=act))
        return y

    def add(self, a, b, act="none"):
        n, c, h, w = self.shape(a)
        y = self.tensor(n, c, h, w)
        self.t.ops.append(Op("add", a, y, in1=b, cin=c, cout=c, act=act))
        return y

    def bn_affine(self, x, act="none"):
        """An unfoldable BatchNorm (one that follows a concatenation) as a per-channel affine: gamma 1, beta 0, mean 0, var 1."""
        n, c, h, w = self.shape(x)
        y = self.tensor(n, c, h, w)
        sc = self.param((c,), "ones", fold=1.0 / math.sqrt(1.0 + BN_EPS))
        sh = self.param((c,), "zeros")
        self.t.ops.append(Op("affine", x, y, scale=sc, shift=sh, cin=c, cout=c, act=act))
        return y

    def scale(self, x, gate, act="none"):
        """y[n,c,h,w] = act(x[n,c,h,w] * gate[n,c]): the channel gate of a squeeze-and-excitation block."""
        n, c, h, w = self.shape(x)
        assert self.shape(gate) == (n, c, 1, 1)
        y = self.tensor(n, c, h, w)
        self.t.ops.append(Op("scale", x, y, in1=gate, cin=c, cout=c, act=act))
        return y

    def concat(self, a, b):
        """Channel concatenation: out[:, :ca] = a, out[:, ca:] = b."""
        n, ca, h, w = self.shape(a)
        nb, cb, hb, wb = self.shape(b)
        assert (n, h, w) == (nb, hb, wb)
        y = self.tensor(n, ca + cb, h, w)
        self.t.ops.append(Op("concat", a, y, in1=b, cin=ca, cout=ca + cb))
        return y

    def avgpool(self, x, k, stride, out=None):
        n, c, h, w = self.shape(x)
        y = self._out(out, (n, c, (h - k) // stride + 1, (w - k) // stride + 1))
        self.t.ops.append(Op("avgpool", x, y, cin=c, cout=c, kh=k, kw=k, stride=stride, pad=0))
        return y

    def act(self, x, act, out=None):
        n, c, h, w = self.shape(x)
        y = self._out(out, (n, c, h, w))
        self.t.ops.append(Op("act", x, y, cin=c, cout=c, act=act))
        return y

    def layernorm(self, x, res=-1, eps=LN_EPS):
        n, c, h, w = self.shape(x)
        y = self.tensor(n, c, h, w)
        g = self.param((c,), "ones")
        b = self.param((c,), "zeros")
        self.t.ops.append(Op("layernorm", x, y, res=res, scale=g, shift=b, cin=c, cout=c, eps=eps))
        return y

    def softmax(self, x):
        n, c, h, w = self.shape(x)
        y = self.tensor(n, c, h, w)
        self.t.ops.append(Op("softmax", x, y, cin=c, cout=c))
        return y

    def attention(self, qkv, heads):
        n, c3, s, _ = self.shape(qkv)
        d_model = c3 // 3
        dh = d_model // heads
        sc = self.tensor(n * heads, s, s, 1)
        self.t.ops.append(Op("bgemm_qk", qkv, sc, cin=dh, cout=s, groups=heads,
                             alpha=1.0 / math.sqrt(dh)))
        p = self.softmax(sc)
        o = self.tensor(n, d_model, s, 1)
        self.t.ops.append(Op("bgemm_pv", p, o, in1=qkv, cin=s, cout=dh, groups=heads))
        return o

    def done(self, x_in, x_out):
        self.t.input, self.t.output = x_in, x_out
        return self.t


# ----------------------------------------------------------------------------
# configuration-1 toy tenants
# ----------------------------------------------------------------------------
def toy_cnn(dtype="f32", batch=1, hw=32):
    b = _B("toy_cnn", dtype, batch)
    x = b.tensor(batch, 3, hw, hw)
    y = b.conv(x, 16, 3, 1, 1, "relu")
    y = b.conv(y, 32, 3, 2, 1, "relu")
    y = b.gavgpool(y)
    y = b.gemm(y, 10, flatten=True)
    return b.done(x, y)


def toy_mlp(dtype="f32", batch=4):
    b = _B("toy_mlp", dtype, batch)
    x = b.tensor(batch, 256, 1, 1)
    y = b.gemm(x, 512, "relu", flatten=True)
    y = b.gemm(y, 10, flatten=True)
    return b.done(x, y)


# ----------------------------------------------------------------------------
# ResNet (He et al. 2016): stem 7x7 s2 p3 -> ReLU -> maxpool 3x3 s2 p1;
# 1x1 projection shortcut only where the shape changes; ReLU after the add;
# bottleneck stride sits on the 3x3.  BatchNorm is folded into the weights.
# ----------------------------------------------------------------------------
def _resnet(name, dtype, batch, hw, blocks, widths, bottleneck, classes, stem=64):
    b = _B(name, dtype, batch)
    x = b.tensor(batch, 3, hw, hw)
    y = b.conv(x, stem, 7, 2, 3, "relu", bn=True)
    y = b.maxpool(y, 3, 2, 1)
    for stage, (nb, wd) in enumerate(zip(blocks, widths)):
        for blk in range(nb):
            stride = 2 if (stage > 0 and blk == 0) else 1
            cin = b.shape(y)[1]
            cout = wd * 4 if bottleneck else wd
            if bottleneck:
                z = b.conv(y, wd, 1, 1, 0, "relu", bn=True)
                z = b.conv(z, wd, 3, stride, 1, "relu", bn=True)
                sc = y if (stride == 1 and cin == cout) else b.conv(y, cout, 1, stride, 0, bn=True)
                y = b.conv(z, cout, 1, 1, 0, "relu", res=sc, bn=True)
            else:
                z = b.conv(y, wd, 3, stride, 1, "relu", bn=True)
                sc = y if (stride == 1 and cin == cout) else b.conv(y, cout, 1, stride, 0, bn=True)
                y = b.conv(z, cout, 3, 1, 1, "relu", res=sc, bn=True)
    y = b.gavgpool(y)
    y = b.gemm(y, classes, flatten=True)
    return b.done(x, y)


def resnet18(dtype="f32", batch=8, hw=224):
    return _resnet("resnet18", dtype, batch, hw, [2, 2, 2, 2], [64, 128, 256, 512], False, 1000)


def resnet50(dtype="bf16", batch=16, hw=224):
    return _resnet("resnet50", dtype, batch, hw, [3, 4, 6, 3], [64, 128, 256, 512], True, 1000)


def resnet34(dtype="f32", batch=8, hw=224):
    return _resnet("resnet34", dtype, batch, hw, [3, 4, 6, 3], [64, 128, 256, 512], False, 1000)


def resnet101(dtype="bf16", batch=8, hw=224):
    return _resnet("resnet101", dtype, batch, hw, [3, 4, 23, 3], [64, 128, 256, 512], True, 1000)


# ----------------------------------------------------------------------------
# AlexNet (Krizhevsky et al. 2012, the single-tower form of Krizhevsky 2014):
# 11x11 s4 p2, 5x5 p2, three 3x3 p1 convolutions with ReLU, 3x3 s2 max-pools
# after the first, second and fifth, flatten in (c,h,w) order, FC-ReLU,
# FC-ReLU, FC.  No normalisation layers.
# ----------------------------------------------------------------------------
def _alexnet(name, dtype, batch, hw, widths, fc, classes):
    c1, c2, c3, c4, c5 = widths
    b = _B(name, dtype, batch)
    x = b.tensor(batch, 3, hw, hw)
    y = b.conv(x, c1, 11, 4, 2, "relu")
    y = b.maxpool(y, 3, 2, 0)
    y = b.conv(y, c2, 5, 1, 2, "relu")
    y = b.maxpool(y, 3, 2, 0)
    y = b.conv(y, c3, 3, 1, 1, "relu")
    y = b.conv(y, c4, 3, 1, 1, "relu")
    y = b.conv(y, c5, 3, 1, 1, "relu")
    y = b.maxpool(y, 3, 2, 0)
    y = b.gemm(y, fc, "relu", flatten=True)
    y = b.gemm(y, fc, "relu", flatten=True)
    y = b.gemm(y, classes, flatten=True)
    return b.done(x, y)


def alexnet(dtype="f32", batch=8, hw=224):
    return _alexnet("alexnet", dtype, batch, hw, (64, 192, 384, 256, 256), 4096, 1000)


# ----------------------------------------------------------------------------
# VGG-16 (Simonyan & Zisserman 2015, configuration D): 13 conv3x3 p1 + ReLU,
# five 2x2 s2 max-pools, flatten in (c,h,w) order, FC-ReLU, FC-ReLU, FC.
# ----------------------------------------------------------------------------
def _vgg(name, dtype, batch, hw, cfg, fc, classes):
    b = _B(name, dtype, batch)
    x = b.tensor(batch, 3, hw, hw)
    y = x
    for v in cfg:
        if v == "M":
            y = b.maxpool(y, 2, 2, 0)
        else:
            y = b.conv(y, v, 3, 1, 1, "relu")
    y = b.gemm(y, fc, "relu", flatten=True)
    y = b.gemm(y, fc, "relu", flatten=True)
    y = b.gemm(y, classes, flatten=True)
    return b.done(x, y)


def vgg16(dtype="bf16", batch=8, hw=224):
    cfg = [64, 64, "M", 128, 128, "M", 256, 256, 256, "M", 512, 512, 512, "M", 512, 512, 512, "M"]
    return _vgg("vgg16", dtype, batch, hw, cfg, 4096, 1000)


# ----------------------------------------------------------------------------
# MobileNetV2 (Sandler et al. 2018), width 1.0: ReLU6 after expand and
# depthwise, linear projection, residual when stride 1 and Cin == Cout.
# ----------------------------------------------------------------------------
def _mbv2(name, dtype, batch, hw, stem, settings, last, classes):
    b = _B(name, dtype, batch)
    x = b.tensor(batch, 3, hw, hw)
    y = b.conv(x, stem, 3, 2, 1, "relu6", bn=True)
    for t, c, n, s in settings:
        for i in range(n):
            stride = s if i == 0 else 1
            cin = b.shape(y)[1]
            z = y
            if t != 1:
                z = b.conv(z, cin * t, 1, 1, 0, "relu6", bn=True)
            hid = b.shape(z)[1]
            z = b.conv(z, hid, 3, stride, 1, "relu6", bn=True, groups=hid)
            res = y if (stride == 1 and cin == c) else -1
            y = b.conv(z, c, 1, 1, 0, "none", res=res, bn=True)
    y = b.conv(y, last, 1, 1, 0, "relu6", bn=True)
    y = b.gavgpool(y)
    y = b.gemm(y, classes, flatten=True)
    return b.done(x, y)


def mobilenetv2(dtype="f32", batch=8, hw=224):
    settings = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
                (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]
    return _mbv2("mobilenetv2", dtype, batch, hw, 32, settings, 1280, 1000)


# ----------------------------------------------------------------------------
# MobileNetV3-Large (Howard et al. 2019, Table 1): inverted residuals with 3x3
# or 5x5 depthwise windows, ReLU or hard-swish, and squeeze-and-excitation
# gates (global mean -> FC-ReLU -> FC-hard-sigmoid -> channel scale) between
# the depthwise and the projection convolution; the gate's inner width is a
# quarter of the expanded width rounded to a multiple of 8.
# ----------------------------------------------------------------------------
# The gate's second FC is drawn this much smaller than He-uniform: without trained weights and without normalisation the
# activations grow to a few hundred, and a hard-sigmoid fed with values of that size is a switch (0 or 1, flipping on a
# rounding error) instead of the smooth gate it is in a trained network; this keeps its input in the linear range.
SE_GATE_FOLD = 1.0 / 32.0


def _round8(v, d=8):
    r = max(d, int(v + d / 2) // d * d)
    return r + d if r < 0.9 * v else r


def _mbv3(name, dtype, batch, hw, stem, settings, last_conv, last_fc, classes):
    b = _B(name, dtype, batch)
    x = b.tensor(batch, 3, hw, hw)
    y = b.conv(x, stem, 3, 2, 1, "hswish", bn=True)
    for k, exp, c, se, nl, s in settings:
        cin = b.shape(y)[1]
        z = y
        if exp != cin:
            z = b.conv(z, exp, 1, 1, 0, nl, bn=True)
        z = b.conv(z, exp, k, s, (k - 1) // 2, nl, bn=True, groups=exp)
        if se:
            g = b.gavgpool(z)
            g = b.gemm(g, _round8(exp // 4), "relu", flatten=True)
            g = b.gemm(g, exp, "hsigmoid", flatten=True, fold=SE_GATE_FOLD)
            z = b.scale(z, g)
        res = y if (s == 1 and cin == c) else -1
        y = b.conv(z, c, 1, 1, 0, "none", res=res, bn=True)
    y = b.conv(y, last_conv, 1, 1, 0, "hswish", bn=True)
    y = b.gavgpool(y)
    y = b.gemm(y, last_fc, "hswish", flatten=True)
    y = b.gemm(y, classes, flatten=True)
    return b.done(x, y)


def mobilenetv3_large(dtype="bf16", batch=8, hw=224):
    R, H = "relu", "hswish"
    settings = [(3, 16, 16, False, R, 1), (3, 64, 24, False, R, 2), (3, 72, 24, False, R, 1),
                (5, 72, 40, True, R, 2), (5, 120, 40, True, R, 1), (5, 120, 40, True, R, 1),
                (3, 240, 80, False, H, 2), (3, 200, 80, False, H, 1), (3, 184, 80, False, H, 1), (3, 184, 80, False, H, 1),
                (3, 480, 112, True, H, 1), (3, 672, 112, True, H, 1),
                (5, 672, 160, True, H, 2), (5, 960, 160, True, H, 1), (5, 960, 160, True, H, 1)]
    return _mbv3("mobilenetv3_large", dtype, batch, hw, 16, settings, 960, 1280, 1000)


# ----------------------------------------------------------------------------
# DenseNet-121 (Huang et al. 2017), growth rate 32, bottleneck width 4, blocks
# of 6/12/24/16 layers.  A dense layer is BN-ReLU-conv1x1-BN-ReLU-conv3x3 and
# its output is concatenated to everything before it; a transition is
# BN-ReLU-conv1x1 (half the channels) and a 2x2 mean pool.  BatchNorms that
# follow a convolution are folded into it; the ones that follow a
# concatenation cannot be and stay as per-channel affine operators.
# The concatenation itself is storage, not work (in_place): a block owns one
# tensor as wide as its last layer's input plus output, the pool in front of
# the block and every layer write their channel windows of it, and a layer
# reads the prefix written so far.  in_place=False spells the same network with
# a concatenation operator that copies.
# ----------------------------------------------------------------------------
def _densenet(name, dtype, batch, hw, growth, blocks, init, bn_size, classes, in_place=True):
    b = _B(name, dtype, batch)
    x = b.tensor(batch, 3, hw, hw)
    y = b.conv(x, init, 7, 2, 3, "relu", bn=True)

    def into_block(src, k, stride, pad, layers):
        """The pool in front of a block (max with padding, mean without); in place, it writes the first window of the block's tensor."""
        pool = (lambda out: b.maxpool(src, k, stride, pad, out=out)) if pad else (lambda out: b.avgpool(src, k, stride, out=out))
        if not in_place:
            return pool(None), None
        n, c, h, w = b.shape(src)
        blk = b.tensor(n, c + layers * growth, (h + 2 * pad - k) // stride + 1, (w + 2 * pad - k) // stride + 1)
        return pool(b.view(blk, 0, c)), blk

    y, blk = into_block(y, 3, 2, 1, blocks[0])
    for bi, layers in enumerate(blocks):
        c = b.shape(y)[1]
        for l in range(layers):
            if in_place and l > 0:
                y = b.view(blk, 0, c)           # everything written so far
            z = b.bn_affine(y, "relu")
            z = b.conv(z, bn_size * growth, 1, 1, 0, "relu", bn=True)
            if in_place:
                b.conv(z, growth, 3, 1, 1, "none", out=b.view(blk, c, growth))
            else:
                y = b.concat(y, b.conv(z, growth, 3, 1, 1, "none"))
            c += growth
        if in_place:
            y = blk                             # all of its windows are written
        if bi + 1 < len(blocks):
            z = b.bn_affine(y, "relu")
            z = b.conv(z, c // 2, 1, 1, 0, "none")
            y, blk = into_block(z, 2, 2, 0, blocks[bi + 1])
    y = b.bn_affine(y, "relu")
    y = b.gavgpool(y)
    y = b.gemm(y, classes, flatten=True)
    return b.done(x, y)


def densenet121(dtype="bf16", batch=8, hw=224):
    return _densenet("densenet121", dtype, batch, hw, 32, [6, 12, 24, 16], 64, 4, 1000)


# ----------------------------------------------------------------------------
# BERT-base-shaped encoder (Devlin et al. 2019), post-LN blocks.  The input is
# the already-embedded sequence; an embedding LayerNorm comes first.
# ----------------------------------------------------------------------------
def _bert(name, dtype, batch, seq, layers, hidden, heads, ffn):
    b = _B(name, dtype, batch)
    x = b.tensor(batch, hidden, seq, 1)
    y = b.layernorm(x)
    for _ in range(layers):
        qkv = b.gemm(y, 3 * hidden)
        a = b.attention(qkv, heads)
        a = b.gemm(a, hidden)
        y = b.layernorm(a, res=y)
        f = b.gemm(y, ffn, "gelu")
        f = b.gemm(f, hidden)
        y = b.layernorm(f, res=y)
    t = b.done(x, y)
    t.input_dist = "normal002"
    return t


def bert_base(dtype="bf16", batch=8, seq=128):
    return _bert("bert_base", dtype, batch, seq, 12, 768, 12, 3072)


# ----------------------------------------------------------------------------
# Reduced members of the same families.  They keep every operator kind, odd
# extents and ragged tile tails, at sizes a direct-loop CPU pass finishes in
# well under a second.
# ----------------------------------------------------------------------------
def small_cnn(dtype="f32", batch=3, hw=20):
    """VGG-shaped: conv/pool/flatten-FC with channel counts that are not tile multiples."""
    return _vgg("small_vgg", dtype, batch, hw, [24, "M", 40, 40, "M"], 72, 10)


def small_alexnet(dtype="f32", batch=3, hw=67):
    """AlexNet-shaped: the 11x11 stride-4 and 5x5 windows, unpadded 3x3 stride-2 pools, odd channel counts."""
    return _alexnet("small_alexnet", dtype, batch, hw, (12, 20, 28, 24, 24), 40, 10)


def small_resnet(dtype="f32", batch=3, hw=40, bottleneck=False):
    return _resnet("small_resnet_b" if bottleneck else "small_resnet", dtype, batch, hw,
                   [1, 2], [16, 24], bottleneck, 10, stem=16)


def small_mbv2(dtype="f32", batch=3, hw=36):
    return _mbv2("small_mbv2", dtype, batch, hw, 8, [(1, 8, 1, 1), (6, 16, 2, 2), (6, 24, 2, 1)], 64, 10)


def small_mbv3(dtype="f32", batch=3, hw=36):
    R, H = "relu", "hswish"
    settings = [(3, 8, 8, False, R, 1), (3, 24, 12, False, R, 2), (5, 40, 12, True, R, 1), (3, 48, 20, True, H, 2),
                (5, 64, 20, True, H, 1)]
    return _mbv3("small_mbv3", dtype, batch, hw, 8, settings, 72, 96, 10)


def small_densenet(dtype="f32", batch=3, hw=40):
    return _densenet("small_densenet", dtype, batch, hw, 8, [2, 3], 12, 2, 10)


def small_bert(dtype="f32", batch=3, seq=24):
    return _bert("small_bert", dtype, batch, seq, 2, 64, 4, 128)


# ----------------------------------------------------------------------------
def materialise(t: Tenant, seed: int, id_offset: int = 0):
    """Draw the tenant's input and parameters.

    Returns (x, params): float32 numpy arrays in logical order.  tensor_id
    ``id_offset`` is the input, parameter p has tensor_id id_offset + p + 1.  In bf16 tenants the input
    and the weights are rounded once to bfloat16 here, so both consumers see
    the same values; biases and normalisation parameters stay fp32.
    """
    shape = t.tensors[t.input]
    if t.input_dist == "normal002":
        x = splitmix64_normal(seed, id_offset, shape, 0.02)
    else:
        x = splitmix64_uniform(seed, id_offset, shape, -1.0, 1.0)
    x = x.astype(np.float32)
    if t.dtype == "bf16":
        x = bf16_round(x)
    is_weight = set(op.w for op in t.ops if op.w >= 0)
    params = []
    for i, p in enumerate(t.params):
        if p.init == "zeros":
            a = np.zeros(p.shape, dtype=np.float64)
        elif p.init == "ones":
            a = np.ones(p.shape, dtype=np.float64)
        elif p.init == "uniform":
            a = splitmix64_uniform(seed, id_offset + i + 1, p.shape, -1.0, 1.0)
        elif p.init == "he_uniform":
            bound = math.sqrt(6.0 / p.fan_in)
            a = splitmix64_uniform(seed, id_offset + i + 1, p.shape, -bound, bound)
        else:
            raise ValueError(p.init)
        a = (a * p.fold).astype(np.float32)
        if t.dtype == "bf16" and i in is_weight:
            a = bf16_round(a)
        params.append(a)
    return x, params


def gemm_macs(t: Tenant) -> int:
    """Multiply-accumulates of the conv / GEMM / attention ops, whole batch."""
    total = 0
    for op in t.ops:
        n, c, h, w = t.tensors[op.out]
        if op.kind in ("conv", "dwconv"):
            total += n * c * h * w * (op.cin // op.groups) * op.kh * op.kw
        elif op.kind == "gemm":
            total += n * c * h * w * op.cin
        elif op.kind in ("bgemm_qk", "bgemm_pv"):
            total += n * c * h * w * op.cin
    return total


def tenant_params(t: Tenant) -> int:
    """Number of conv / GEMM weights and biases and of per-channel affine parameters."""
    total = 0
    for op in t.ops:
        if op.kind in ("conv", "dwconv", "gemm"):
            total += int(np.prod(t.params[op.w].shape)) + int(np.prod(t.params[op.bias].shape))
        elif op.kind == "affine":
            total += int(np.prod(t.params[op.scale].shape)) + int(np.prod(t.params[op.shift].shape))
    return total
