"""Seeded synthetic inputs and layer-shape recipes.

Serves both the GPU library's callers (tests, bench) and the CPU oracle's
callers; holds none of the method's arithmetic.  Shapes follow the networks of
Section IV-A of arXiv 2006.09791 (WRN-40-2 for CIFAR-sized 32x32 inputs,
ResNet-34 and MobileNet-style depthwise layers for 224x224 inputs); values are
synthetic: inputs uniform in [-1, 1), weights normal with std sqrt(2 / fan_in),
fan_in = (Cin/g) * KH * KW.
"""
from collections import namedtuple

import numpy as np

# One step of a layer chain.  Buffers are referred to by index.
#   op    : "conv" | "maxpool" | "add" | "relu"
#   src   : input buffer; src2: second operand ("add") or residual added to the
#           convolution result before the optional ReLU ("conv"), -1 if none
#   relu  : apply max(., 0) to the result of a conv / add
#   wid   : index into the chain's weight list (conv only)
Layer = namedtuple(
    "Layer", "op src src2 dst N Cin H W Cout KH KW stride pad groups relu wid")

ConvShape = namedtuple("ConvShape", "N Cin H W Cout KH KW stride pad groups")


def out_size(size, k, stride, pad):
    return (size + 2 * pad - k) // stride + 1


def conv_macs(s):
    """MAC count of one layer (Eq. 2 of the paper)."""
    ho, wo = out_size(s.H, s.KH, s.stride, s.pad), out_size(s.W, s.KW, s.stride, s.pad)
    return s.N * s.Cin * s.Cout * s.KH * s.KW * ho * wo // s.groups


def make_seed(config_id, layer_index, groups):
    return (1000003 * config_id + 1009 * layer_index + groups) % (2 ** 31 - 1)


def make_input(shape, seed):
    rng = np.random.default_rng(seed)
    return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)


def make_weight(Cout, CPG, KH, KW, seed):
    rng = np.random.default_rng(seed + 7919)
    std = np.sqrt(2.0 / (CPG * KH * KW))
    return (rng.standard_normal(size=(Cout, CPG, KH, KW)) * std).astype(np.float32)


def round_to_bf16(a):
    """fp32 -> nearest-even bf16.  Returns (uint16 bit patterns, the same
    values widened back to fp32)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)
    back = (r.astype(np.uint32) << 16).view(np.float32)
    return r, back.reshape(a.shape)


# ----------------------------------------------------------------------------
# Single layers
# ----------------------------------------------------------------------------
def config1():
    """Small smoke / parity case: 64 -> 64 channels, 32x32, 3x3, g = 4."""
    return ConvShape(1, 64, 32, 32, 64, 3, 3, 1, 1, 4)


def wrn_grouped_shapes(N, g):
    """The five distinct grouped 3x3 layers of the WRN-40-2-style stack."""
    return [
        ConvShape(N, 32, 32, 32, 32, 3, 3, 1, 1, g),
        ConvShape(N, 32, 32, 32, 64, 3, 3, 2, 1, g),
        ConvShape(N, 64, 16, 16, 64, 3, 3, 1, 1, g),
        ConvShape(N, 64, 16, 16, 128, 3, 3, 2, 1, g),
        ConvShape(N, 128, 8, 8, 128, 3, 3, 1, 1, g),
    ]


def resnet34_grouped_shapes(N, g):
    """The seven distinct grouped 3x3 layers of the ResNet-34-shaped stack."""
    return [
        ConvShape(N, 64, 56, 56, 64, 3, 3, 1, 1, g),
        ConvShape(N, 64, 56, 56, 128, 3, 3, 2, 1, g),
        ConvShape(N, 128, 28, 28, 128, 3, 3, 1, 1, g),
        ConvShape(N, 128, 28, 28, 256, 3, 3, 2, 1, g),
        ConvShape(N, 256, 14, 14, 256, 3, 3, 1, 1, g),
        ConvShape(N, 256, 14, 14, 512, 3, 3, 2, 1, g),
        ConvShape(N, 512, 7, 7, 512, 3, 3, 1, 1, g),
    ]


DEPTHWISE_CH_HW = [(32, 112), (64, 112), (128, 56), (256, 28), (512, 14), (1024, 7)]


def depthwise_pairs(N=1):
    """MobileNet-shaped (depthwise 3x3, pointwise 1x1 C -> 2C) layer pairs."""
    pairs = []
    for C, hw in DEPTHWISE_CH_HW:
        for stride in (1, 2):
            dw = ConvShape(N, C, hw, hw, C, 3, 3, stride, 1, C)
            ho = out_size(hw, 3, stride, 1)
            pw = ConvShape(N, C, ho, ho, 2 * C, 1, 1, 1, 0, 1)
            pairs.append((dw, pw))
    return pairs


# ----------------------------------------------------------------------------
# Layer chains
# ----------------------------------------------------------------------------
class Chain:
    """A list of Layer steps plus the buffers and weights they refer to."""

    def __init__(self, name, input_shape):
        self.name = name
        self.input_shape = tuple(input_shape)
        self.layers = []
        self.weight_shapes = []      # (Cout, CPG, KH, KW) per conv
        self.weight_groups = []
        self.buf_elems = [int(np.prod(input_shape))]   # buffer 0 = chain input
        self.out_buf = 0
        self.out_shape = tuple(input_shape)

    def _need(self, buf, elems):
        while len(self.buf_elems) <= buf:
            self.buf_elems.append(0)
        self.buf_elems[buf] = max(self.buf_elems[buf], int(elems))

    def conv(self, src, dst, N, Cin, H, W, Cout, k, stride, pad, groups,
             relu=False, residual=-1):
        ho, wo = out_size(H, k, stride, pad), out_size(W, k, stride, pad)
        wid = len(self.weight_shapes)
        self.weight_shapes.append((Cout, Cin // groups, k, k))
        self.weight_groups.append(groups)
        self.layers.append(Layer("conv", src, residual, dst, N, Cin, H, W, Cout,
                                 k, k, stride, pad, groups, bool(relu), wid))
        self._need(dst, N * Cout * ho * wo)
        self.out_buf, self.out_shape = dst, (N, Cout, ho, wo)
        return ho, wo

    def maxpool(self, src, dst, N, C, H, W, k=3, stride=2, pad=1):
        ho, wo = out_size(H, k, stride, pad), out_size(W, k, stride, pad)
        self.layers.append(Layer("maxpool", src, -1, dst, N, C, H, W, C, k, k,
                                 stride, pad, 1, False, -1))
        self._need(dst, N * C * ho * wo)
        self.out_buf, self.out_shape = dst, (N, C, ho, wo)
        return ho, wo

    def macs(self):
        return sum(conv_macs(ConvShape(l.N, l.Cin, l.H, l.W, l.Cout, l.KH, l.KW,
                                       l.stride, l.pad, l.groups))
                   for l in self.layers if l.op == "conv")

    def make_weights(self, config_id):
        return [make_weight(*shp, seed=make_seed(config_id, i, g))
                for i, (shp, g) in enumerate(zip(self.weight_shapes,
                                                 self.weight_groups))]


def _conv3(ch, src, dst, tmp, N, cin, hw, cout, stride, g, pointwise, relu, residual=-1):
    """One 3x3 convolution of a basic block.  pointwise = False: a grouped 3x3 cin -> cout.
    pointwise = True: the replacement the paper trains (Section IV-A), a grouped 3x3
    cin -> cin into `tmp` followed by a 1x1 cin -> cout that mixes the groups; the block's
    ReLU and residual go on the 1x1."""
    if not pointwise:
        return ch.conv(src, dst, N, cin, hw, hw, cout, 3, stride, 1, g, relu=relu, residual=residual)[0]
    ho, _ = ch.conv(src, tmp, N, cin, hw, hw, cin, 3, stride, 1, g)
    ch.conv(tmp, dst, N, cin, ho, ho, cout, 1, 1, 0, 1, relu=relu, residual=residual)
    return ho


def _basic_stage(ch, cur, N, cin, cout, hw, blocks, g, entry_stride, pointwise=False):
    """Residual stage of basic blocks (two grouped 3x3 convs each).  Buffers
    1..4 rotate (5 is the grouped result in the pointwise form); `cur` holds the
    stage input.  Returns (buffer, spatial)."""
    for b in range(blocks):
        free = [i for i in (1, 2, 3, 4) if i != cur]
        t, sc, out = free[0], free[1], free[2]
        if b == 0 and (entry_stride != 1 or cin != cout):
            ho, _ = ch.conv(cur, sc, N, cin, hw, hw, cout, 1, entry_stride, 0, 1)
            _conv3(ch, cur, t, 5, N, cin, hw, cout, entry_stride, g, pointwise, True)
            _conv3(ch, t, out, 5, N, cout, ho, cout, 1, g, pointwise, True, residual=sc)
            hw = ho
        else:
            _conv3(ch, cur, t, 5, N, cout, hw, cout, 1, g, pointwise, True)
            _conv3(ch, t, out, 5, N, cout, hw, cout, 1, g, pointwise, True, residual=cur)
        cur = out
    return cur, hw


def wrn_chain(N, g, pointwise=False):
    """WRN-40-2-style CIFAR stack, every 3x3 conv after the stem grouped.  pointwise = True
    is the form of the paper's trained networks (Section IV-A): each of those convolutions
    becomes a grouped 3x3 a -> a plus a 1x1 a -> b."""
    ch = Chain(f"wrn40x2{'pw' if pointwise else ''}_g{g}_n{N}", (N, 3, 32, 32))
    ch.conv(0, 1, N, 3, 32, 32, 32, 3, 1, 1, 1, relu=True)
    cur, hw = 1, 32
    cur, hw = _basic_stage(ch, cur, N, 32, 32, hw, 6, g, 1, pointwise)
    cur, hw = _basic_stage(ch, cur, N, 32, 64, hw, 6, g, 2, pointwise)
    cur, hw = _basic_stage(ch, cur, N, 64, 128, hw, 6, g, 2, pointwise)
    return ch


def resnet34_chain(N, g, pointwise=False):
    """ResNet-34-shaped ImageNet stack: 7x7 s2 stem, 3x3 s2 max pool, then
    3/4/6/3 basic blocks with every 3x3 conv grouped (pointwise = True: each followed
    by a 1x1, as in wrn_chain)."""
    ch = Chain(f"resnet34{'pw' if pointwise else ''}_g{g}_n{N}", (N, 3, 224, 224))
    ho, _ = ch.conv(0, 1, N, 3, 224, 224, 64, 7, 2, 3, 1, relu=True)
    ho, _ = ch.maxpool(1, 2, N, 64, ho, ho)
    cur, hw = 2, ho
    cur, hw = _basic_stage(ch, cur, N, 64, 64, hw, 3, g, 1, pointwise)
    cur, hw = _basic_stage(ch, cur, N, 64, 128, hw, 4, g, 2, pointwise)
    cur, hw = _basic_stage(ch, cur, N, 128, 256, hw, 6, g, 2, pointwise)
    cur, hw = _basic_stage(ch, cur, N, 256, 512, hw, 3, g, 2, pointwise)
    return ch


# (channels in, channels out, stride) of the 13 blocks of a MobileNet-shaped ImageNet body
MOBILENET_BLOCKS = [(32, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1), (256, 512, 2),
                    (512, 512, 1), (512, 512, 1), (512, 512, 1), (512, 512, 1), (512, 512, 1),
                    (512, 1024, 2), (1024, 1024, 1)]


def mobilenet_chain(N, g=None, hw=224):
    """MobileNet-shaped stack in the form of the paper's networks (Section IV-A): a 3x3
    stride-2 stem 3 -> 32, then 13 blocks of a grouped 3x3 convolution a -> a followed by
    a pointwise 1x1 convolution a -> b.  g = None is the depthwise extreme G(N) (g = a);
    otherwise every 3x3 convolution of the body has g groups.  Two activation buffers
    alternate, so the 3x3 result of a block is overwritten two steps later."""
    tag = "dw" if g is None else f"g{g}"
    ch = Chain(f"mobilenet_{tag}_n{N}", (N, 3, hw, hw))
    h, _ = ch.conv(0, 1, N, 3, hw, hw, 32, 3, 2, 1, 1, relu=True)
    cur = 1
    for a, b_, s in MOBILENET_BLOCKS:
        mid, out = (2, 3) if cur == 1 else ((1, 3) if cur == 2 else (1, 2))
        ho, _ = ch.conv(cur, mid, N, a, h, h, a, 3, s, 1, a if g is None else g, relu=True)
        ch.conv(mid, out, N, a, ho, ho, b_, 1, 1, 0, 1, relu=True)
        cur, h = out, ho
    return ch


# (expansion t, channels out, repeats, stride of the first repeat) of the bottleneck stages of the
# MobileNetV2 ImageNet definition (its architecture table), between a 3x3 stride-2 stem 3 -> 32 and
# a final 1x1 320 -> 1280
MOBILENETV2_STAGES = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1),
                      (6, 160, 3, 2), (6, 320, 1, 1)]


def mobilenetv2_chain(N, g=None, hw=224):
    """MobileNetV2-shaped stack (Section IV-A's third network): inverted-residual blocks of a
    1x1 expansion a -> t*a, a 3x3 convolution t*a -> t*a with g groups (g = None: the depthwise
    original, G(N)) and a linear 1x1 projection t*a -> b, with the block input added where
    stride 1 keeps the shape.  The activation is the chain's ReLU (the original clips at 6;
    the shapes, not the clip, are what is timed).  Buffers 1..4 rotate."""
    tag = "dw" if g is None else f"g{g}"
    ch = Chain(f"mobilenetv2_{tag}_n{N}", (N, 3, hw, hw))
    h, _ = ch.conv(0, 1, N, 3, hw, hw, 32, 3, 2, 1, 1, relu=True)
    cur, a = 1, 32
    for t, c, n, s in MOBILENETV2_STAGES:
        for i in range(n):
            stride = s if i == 0 else 1
            e, d, out = [k for k in (1, 2, 3, 4) if k != cur][:3]
            m = a * t
            src = cur
            if t != 1:
                ch.conv(cur, e, N, a, h, h, m, 1, 1, 0, 1, relu=True)
                src = e
            ho, _ = ch.conv(src, d, N, m, h, h, m, 3, stride, 1, m if g is None else g, relu=True)
            ch.conv(d, out, N, m, ho, ho, c, 1, 1, 0, 1, residual=cur if (stride == 1 and a == c) else -1)
            cur, a, h = out, c, ho
    e = 1 if cur != 1 else 2
    ch.conv(cur, e, N, a, h, h, 1280, 1, 1, 0, 1, relu=True)
    return ch


def mobilenet_dw_chain(N, C, hw, stride):
    """Depthwise 3x3 (g = C) followed by a pointwise 1x1 C -> 2C."""
    ch = Chain(f"dw_c{C}_hw{hw}_s{stride}_n{N}", (N, C, hw, hw))
    ho, _ = ch.conv(0, 1, N, C, hw, hw, C, 3, stride, 1, C, relu=True)
    ch.conv(1, 2, N, C, ho, ho, 2 * C, 1, 1, 0, 1, relu=True)
    return ch
