"""Layer tables for the synthetic workloads.

A net is an ordered list of `Op`s over numbered activation buffers.  Buffer 0 is
the net input; the last op's `dst` is the net output.  The tables only carry
shapes, strides, sparsities and buffer wiring -- no arithmetic.

ResNet-50 layout (the paper's Table 2 names the model but not its layer
details; the standard 3/4/6/3 bottleneck ladder is used): conv1 7x7/2, maxpool
3x3/2, 16 bottlenecks (1x1 reduce, 3x3, 1x1 expand; x4 expansion; mid channels
64/128/256/512), projection 1x1 shortcuts on the first block of each stage,
stride 2 placed on the 3x3 (and on the projection) of the first block of stages
3-5, global average pool, FC 2048->1000.  That is 1 + 16*3 + 4 = 53 convs.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

from .gen import activation, bias_vector, conv_out_size, embed_filter, pruned_weights


@dataclass(frozen=True)
class Op:
    kind: str              # "conv" | "dwconv" (depthwise; cin == cout) | "fc" | "maxpool" | "avgpool" (global)
                           # | "avgpool2d" (k x k windows) | "concat"
    name: str
    src: int
    dst: int
    cin: int = 0
    cout: int = 0
    k: int = 1             # square kernel / pool window
    stride: int = 1
    pad: int = 0
    sparsity: float = 0.0
    relu: bool = False
    res: int = -1          # buffer added before the activation, -1 = none
    kh: int = 0            # rectangular filter kh x kw centred in the k x k one (0 = square k x k)
    kw: int = 0
    srcs: Tuple[int, ...] = ()   # "concat": the buffers stacked along the channel axis, in order


def single_conv_ops(cin=64, cout=64, k=3, stride=1, pad=1, sparsity=0.9, relu=True) -> List[Op]:
    return [Op("conv", "conv", 0, 1, cin, cout, k, stride, pad, sparsity, relu)]


def bottleneck_conv2x_ops(sparsity: float = 0.85) -> List[Op]:
    """conv2_x identity bottleneck: 1x1 256->64, 3x3 64->64 pad 1, 1x1 64->256 + input, ReLU."""
    return [
        Op("conv", "a_1x1", 0, 1, 256, 64, 1, 1, 0, sparsity, True),
        Op("conv", "b_3x3", 1, 2, 64, 64, 3, 1, 1, sparsity, True),
        Op("conv", "c_1x1", 2, 3, 64, 256, 1, 1, 0, sparsity, True, res=0),
    ]


def resnet50_ops(s_conv1: float = 0.0, s_3x3: float = 0.8, s_1x1: float = 0.9,
                 s_fc: float = 0.9, stride_on_1x1: bool = False,
                 uniform: float | None = None) -> List[Op]:
    if uniform is not None:
        s_conv1 = s_3x3 = s_1x1 = s_fc = uniform
    ops: List[Op] = []
    ops.append(Op("conv", "conv1", 0, 1, 3, 64, 7, 2, 3, s_conv1, True))
    ops.append(Op("maxpool", "pool1", 1, 2, k=3, stride=2, pad=1))
    cur, other = 2, 3
    t1, t2, tp = 4, 5, 6
    cin = 64
    for stage, (nblocks, mid) in enumerate([(3, 64), (4, 128), (6, 256), (3, 512)], start=2):
        for b in range(nblocks):
            first = b == 0
            stride = 2 if (first and stage > 2) else 1
            cout = mid * 4
            sa, sb = (stride, 1) if stride_on_1x1 else (1, stride)
            tag = f"conv{stage}_{b + 1}"
            ops.append(Op("conv", tag + "a", cur, t1, cin, mid, 1, sa, 0, s_1x1, True))
            ops.append(Op("conv", tag + "b", t1, t2, mid, mid, 3, sb, 1, s_3x3, True))
            if first:
                ops.append(Op("conv", tag + "p", cur, tp, cin, cout, 1, stride, 0, s_1x1, False))
                res = tp
            else:
                res = cur
            ops.append(Op("conv", tag + "c", t2, other, mid, cout, 1, 1, 0, s_1x1, True, res=res))
            cur, other = other, cur
            cin = cout
    ops.append(Op("avgpool", "gap", cur, 7))
    ops.append(Op("fc", "fc", 7, 8, 2048, 1000, sparsity=s_fc, relu=False))
    return ops


def vgg16_ops(s_conv: float = 0.9, s_fc: float = 0.96) -> List[Op]:
    cfg = [64, 64, "M", 128, 128, "M", 256, 256, 256, "M", 512, 512, 512, "M", 512, 512, 512, "M"]
    ops: List[Op] = []
    cur, cin, i = 0, 3, 0
    nxt = 1
    for v in cfg:
        if v == "M":
            ops.append(Op("maxpool", f"pool{len(ops)}", cur, nxt, k=2, stride=2, pad=0))
        else:
            i += 1
            ops.append(Op("conv", f"conv{i}", cur, nxt, cin, int(v), 3, 1, 1, s_conv, True))
            cin = int(v)
        cur, nxt = nxt, (1 if nxt == 2 else 2)
    ops.append(Op("fc", "fc1", cur, 3, 512 * 7 * 7, 4096, sparsity=s_fc, relu=True))
    ops.append(Op("fc", "fc2", 3, 4, 4096, 4096, sparsity=s_fc, relu=True))
    ops.append(Op("fc", "fc3", 4, 5, 4096, 1000, sparsity=s_fc, relu=False))
    return ops


def mobilenet_v1_ops(s_conv1: float = 0.0, s_dw: float = 0.0, s_pw: float = 0.8,
                     s_fc: float = 0.9) -> List[Op]:
    """MobileNet-V1 at width 1.0 and 224x224 input (the paper's Table 2 names the model):
    a 3x3/2 convolution to 32 channels, 13 depthwise-separable blocks (3x3 depthwise +
    1x1 pointwise, each followed by batch-norm + ReLU, folded here into bias + ReLU; the
    blocks' output channels and depthwise strides below are the published ladder), global
    average pool, FC 1024->1000.  The pointwise layers carry nearly all the weights and are
    the pruned ones; depthwise filters (9 weights per channel) stay dense by default."""
    ladder = [(64, 1), (128, 2), (128, 1), (256, 2), (256, 1), (512, 2), (512, 1), (512, 1),
              (512, 1), (512, 1), (512, 1), (1024, 2), (1024, 1)]
    ops: List[Op] = [Op("conv", "conv1", 0, 1, 3, 32, 3, 2, 1, s_conv1, True)]
    cur, cin = 1, 32
    for i, (cout, stride) in enumerate(ladder, start=1):
        mid = 2 if cur == 1 else (1 if cur == 3 else 3)
        nxt = ({1, 2, 3} - {cur, mid}).pop()
        ops.append(Op("dwconv", f"dw{i}", cur, mid, cin, cin, 3, stride, 1, s_dw, True))
        ops.append(Op("conv", f"pw{i}", mid, nxt, cin, cout, 1, 1, 0, s_pw, True))
        cur, cin = nxt, cout
    ops.append(Op("avgpool", "gap", cur, 4))
    ops.append(Op("fc", "fc", 4, 5, 1024, 1000, sparsity=s_fc, relu=False))
    return ops


def mobilenet_v2_ops(s_conv1: float = 0.0, s_dw: float = 0.0, s_pw: float = 0.8,
                     s_fc: float = 0.9) -> List[Op]:
    """MobileNet-V2 at width 1.0 and 224x224 input (named in the paper's Table 2): a 3x3/2
    convolution to 32 channels, 17 inverted-residual blocks -- 1x1 expansion by t (absent
    when t = 1) + ReLU, 3x3 depthwise + ReLU, linear 1x1 projection, plus the block input when
    the stride is 1 and the channel counts agree -- in the published (t, c, n, s) ladder, a
    1x1 convolution to 1280 channels, global average pool, FC 1280->1000.  The published
    network clips activations at 6; the layers here use plain ReLU (the fused epilogue the
    paper describes)."""
    ladder = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2),
              (6, 320, 1, 1)]
    ops: List[Op] = [Op("conv", "conv1", 0, 1, 3, 32, 3, 2, 1, s_conv1, True)]
    cur, cin, blk = 1, 32, 0
    for t, cout, reps, stride in ladder:
        for r in range(reps):
            blk += 1
            st = stride if r == 0 else 1
            free = [b for b in (1, 2, 3, 4) if b != cur]
            mid = cin * t
            src = cur
            if t != 1:
                ops.append(Op("conv", f"b{blk}_expand", src, free[0], cin, mid, 1, 1, 0, s_pw, True))
                src = free[0]
            ops.append(Op("dwconv", f"b{blk}_dw", src, free[1], mid, mid, 3, st, 1, s_dw, True))
            res = cur if (st == 1 and cin == cout) else -1
            ops.append(Op("conv", f"b{blk}_project", free[1], free[2], mid, cout, 1, 1, 0, s_pw, False, res=res))
            cur, cin = free[2], cout
    last = 1 if cur != 1 else 2
    ops.append(Op("conv", "conv_last", cur, last, cin, 1280, 1, 1, 0, s_pw, True))
    ops.append(Op("avgpool", "gap", last, 5))
    ops.append(Op("fc", "fc", 5, 6, 1280, 1000, sparsity=s_fc, relu=False))
    return ops


def factorized_7x7_branch_ops(cin: int = 768, mid: int = 128, cout: int = 192, sparsity: float = 0.8) -> List[Op]:
    """The deepest branch of an Inception-V3 17x17 module (the paper's Table 2 names the model):
    1x1, then 7x1, 1x7, 7x1, 1x7 filters with "same" padding (the published factorisation of a
    7x7 convolution).  The rectangular filters are carried centred in 7x7 banks with padding 3."""
    ops = [Op("conv", "b_1x1", 0, 1, cin, mid, 1, 1, 0, sparsity, True)]
    shapes = [(7, 1), (1, 7), (7, 1), (1, 7)]
    cur, c = 1, mid
    for i, (kh, kw) in enumerate(shapes):
        co = cout if i == len(shapes) - 1 else mid
        nxt = 2 if cur == 1 else 1
        ops.append(Op("conv", "b_%dx%d_%d" % (kh, kw, i + 1), cur, nxt, c, co, 7, 1, 3, sparsity, True, kh=kh, kw=kw))
        cur, c = nxt, co
    return ops


def inception_v3_ops(s_conv1: float = 0.0, s_conv: float = 0.8, s_fc: float = 0.9) -> List[Op]:
    """Inception-V3 at 299x299 input (named in the paper's Table 2; the published module
    ladder without the auxiliary head): a stem of five convolutions and two max pools, three
    35x35 modules (1x1 / 5x5 / double 3x3 / pooled 1x1 branches), a grid reduction, four 17x17
    modules whose 7x7 convolutions are factorised into 1x7 and 7x1 ones, a second reduction,
    two 8x8 modules with 1x3 / 3x1 splits, global average pool, FC 2048->1000: 94
    convolutions.  Every branch output is stacked along the channel axis by a "concat" op;
    rectangular filters are carried centred in square banks (see `embed_filter`).  Each
    convolution stands for convolution + folded batch-norm + ReLU."""
    ops: List[Op] = []
    fresh = iter(range(1, 10000))

    def conv(name, src, cin, cout, k=1, stride=1, pad=0, kh=0, kw=0, first=False):
        dst = next(fresh)
        ops.append(Op("conv", name, src, dst, cin, cout, k, stride, pad, s_conv1 if first else s_conv, True,
                      kh=kh, kw=kw))
        return dst

    def pool(kind, name, src, k, stride, pad):
        dst = next(fresh)
        ops.append(Op(kind, name, src, dst, k=k, stride=stride, pad=pad))
        return dst

    def cat(name, parts):
        dst = next(fresh)
        ops.append(Op("concat", name, parts[0], dst, srcs=tuple(parts)))
        return dst

    x = conv("stem1", 0, 3, 32, 3, 2, 0, first=True)
    x = conv("stem2", x, 32, 32, 3, 1, 0)
    x = conv("stem3", x, 32, 64, 3, 1, 1)
    x = pool("maxpool", "stem_pool1", x, 3, 2, 0)
    x = conv("stem4", x, 64, 80, 1)
    x = conv("stem5", x, 80, 192, 3, 1, 0)
    x = pool("maxpool", "stem_pool2", x, 3, 2, 0)
    c = 192
    for i, pf in enumerate([32, 64, 64]):                      # 35 x 35 modules
        t = "a%d_" % (i + 1)
        b1 = conv(t + "1x1", x, c, 64)
        b5 = conv(t + "5x5b", conv(t + "5x5a", x, c, 48), 48, 64, 5, 1, 2)
        b3 = conv(t + "3x3a", x, c, 64)
        b3 = conv(t + "3x3b", b3, 64, 96, 3, 1, 1)
        b3 = conv(t + "3x3c", b3, 96, 96, 3, 1, 1)
        bp = conv(t + "pool1x1", pool("avgpool2d", t + "pool", x, 3, 1, 1), c, pf)
        x = cat(t + "cat", [b1, b5, b3, bp])
        c = 64 + 64 + 96 + pf
    t = "b_"                                                    # 35 -> 17 reduction
    b3 = conv(t + "3x3", x, c, 384, 3, 2, 0)
    bd = conv(t + "dbl_a", x, c, 64)
    bd = conv(t + "dbl_b", bd, 64, 96, 3, 1, 1)
    bd = conv(t + "dbl_c", bd, 96, 96, 3, 2, 0)
    bp = pool("maxpool", t + "pool", x, 3, 2, 0)
    x = cat(t + "cat", [b3, bd, bp])
    c = 384 + 96 + c
    for i, c7 in enumerate([128, 160, 160, 192]):               # 17 x 17 modules
        t = "c%d_" % (i + 1)
        b1 = conv(t + "1x1", x, c, 192)
        b7 = conv(t + "7a", x, c, c7)
        b7 = conv(t + "7b", b7, c7, c7, 7, 1, 3, kh=1, kw=7)
        b7 = conv(t + "7c", b7, c7, 192, 7, 1, 3, kh=7, kw=1)
        bd = conv(t + "dbl_a", x, c, c7)
        bd = conv(t + "dbl_b", bd, c7, c7, 7, 1, 3, kh=7, kw=1)
        bd = conv(t + "dbl_c", bd, c7, c7, 7, 1, 3, kh=1, kw=7)
        bd = conv(t + "dbl_d", bd, c7, c7, 7, 1, 3, kh=7, kw=1)
        bd = conv(t + "dbl_e", bd, c7, 192, 7, 1, 3, kh=1, kw=7)
        bp = conv(t + "pool1x1", pool("avgpool2d", t + "pool", x, 3, 1, 1), c, 192)
        x = cat(t + "cat", [b1, b7, bd, bp])
        c = 768
    t = "d_"                                                    # 17 -> 8 reduction
    b3 = conv(t + "3x3b", conv(t + "3x3a", x, c, 192), 192, 320, 3, 2, 0)
    b7 = conv(t + "7a", x, c, 192)
    b7 = conv(t + "7b", b7, 192, 192, 7, 1, 3, kh=1, kw=7)
    b7 = conv(t + "7c", b7, 192, 192, 7, 1, 3, kh=7, kw=1)
    b7 = conv(t + "7d", b7, 192, 192, 3, 2, 0)
    bp = pool("maxpool", t + "pool", x, 3, 2, 0)
    x = cat(t + "cat", [b3, b7, bp])
    c = 320 + 192 + c
    for i in range(2):                                          # 8 x 8 modules
        t = "e%d_" % (i + 1)
        b1 = conv(t + "1x1", x, c, 320)
        b3 = conv(t + "3a", x, c, 384)
        b3a = conv(t + "3b", b3, 384, 384, 3, 1, 1, kh=1, kw=3)
        b3b = conv(t + "3c", b3, 384, 384, 3, 1, 1, kh=3, kw=1)
        bd = conv(t + "dbl_a", x, c, 448)
        bd = conv(t + "dbl_b", bd, 448, 384, 3, 1, 1)
        bda = conv(t + "dbl_c", bd, 384, 384, 3, 1, 1, kh=1, kw=3)
        bdb = conv(t + "dbl_d", bd, 384, 384, 3, 1, 1, kh=3, kw=1)
        bp = conv(t + "pool1x1", pool("avgpool2d", t + "pool", x, 3, 1, 1), c, 192)
        x = cat(t + "cat", [b1, b3a, b3b, bda, bdb, bp])
        c = 320 + 768 + 768 + 192
    g = next(fresh)
    ops.append(Op("avgpool", "gap", x, g))
    ops.append(Op("fc", "fc", g, next(fresh), 2048, 1000, sparsity=s_fc, relu=False))
    return ops


def buffer_shapes(ops: Sequence[Op], input_shape: Tuple[int, int, int, int]) -> Dict[int, Tuple[int, ...]]:
    """Largest shape each buffer id takes, by walking the op list (shape inference only)."""
    cur: Dict[int, Tuple[int, ...]] = {0: tuple(input_shape)}
    biggest: Dict[int, Tuple[int, ...]] = {0: tuple(input_shape)}
    for op in ops:
        s = cur[op.src]
        if op.kind == "conv":
            n, c, h, w = s
            assert c == op.cin, (op, s)
            o = (n, op.cout, conv_out_size(h, op.k, op.stride, op.pad),
                 conv_out_size(w, op.k, op.stride, op.pad))
        elif op.kind == "dwconv":
            n, c, h, w = s
            assert c == op.cin == op.cout, (op, s)
            o = (n, c, conv_out_size(h, op.k, op.stride, op.pad),
                 conv_out_size(w, op.k, op.stride, op.pad))
        elif op.kind == "maxpool":
            n, c, h, w = s
            o = (n, c, conv_out_size(h, op.k, op.stride, op.pad),
                 conv_out_size(w, op.k, op.stride, op.pad))
        elif op.kind == "avgpool2d":
            n, c, h, w = s
            o = (n, c, conv_out_size(h, op.k, op.stride, op.pad),
                 conv_out_size(w, op.k, op.stride, op.pad))
        elif op.kind == "concat":
            parts = [cur[b] for b in op.srcs]
            assert all(p[0] == parts[0][0] and p[2:] == parts[0][2:] for p in parts), (op, parts)
            o = (parts[0][0], sum(p[1] for p in parts), parts[0][2], parts[0][3])
        elif op.kind == "avgpool":
            n, c, h, w = s
            o = (n, c, 1, 1)
        elif op.kind == "fc":
            n = s[0]
            assert int(np.prod(s[1:])) == op.cin, (op, s)
            o = (n, op.cout, 1, 1)
        else:
            raise ValueError(op.kind)
        cur[op.dst] = o
        if op.dst not in biggest or np.prod(o) > np.prod(biggest[op.dst]):
            biggest[op.dst] = o
    return biggest


def net_tensors(ops: Sequence[Op], config: str, input_shape, input_relu: bool = False,
                mask: str = "magnitude"):
    """Seeded input, pruned weights and biases for every conv/fc op of a net.

    Returns (x, weights, biases): weights[i] / biases[i] are None for pool ops.
    """
    x = activation(input_shape, config, 0, relu=input_relu)
    weights, biases = [], []
    for i, op in enumerate(ops):
        if op.kind == "conv" and (op.kh or op.kw):
            w = pruned_weights(op.cout, op.cin, op.kh or op.k, op.kw or op.k, op.sparsity, config, i + 1, mask)
            weights.append(embed_filter(w, op.k))
            biases.append(bias_vector(op.cout, config, i + 1))
        elif op.kind == "conv":
            weights.append(pruned_weights(op.cout, op.cin, op.k, op.k, op.sparsity, config, i + 1, mask))
            biases.append(bias_vector(op.cout, config, i + 1))
        elif op.kind == "dwconv":
            weights.append(pruned_weights(op.cout, 1, op.k, op.k, op.sparsity, config, i + 1, mask))
            biases.append(bias_vector(op.cout, config, i + 1))
        elif op.kind == "fc":
            weights.append(pruned_weights(op.cout, op.cin, 1, 1, op.sparsity, config, i + 1, mask))
            biases.append(bias_vector(op.cout, config, i + 1))
        else:
            weights.append(None)
            biases.append(None)
    return x, weights, biases
