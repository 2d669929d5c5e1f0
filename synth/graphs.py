"""Layer-graph descriptors of the model families the paper evaluates.

A graph is a list of nodes in execution order.  Every node is one weighted
layer (convolution, depthwise convolution, or the classifier that follows a
global average pool) described by 13 int32 fields, the same record the C
boundary takes:

    kind, cin, cout, kh, kw, stride, pad, hin, win, input, residual, act, scheme_slot

``input``/``residual`` are node indices (-1 = network input / no residual);
``scheme_slot`` is the position of the layer inside a bit-width scheme
``q = (q_1 .. q_L)`` (paper, Problem Formulation), or -1 for a layer that is
never part of a scheme (ResNet projection shortcuts stay FP32).

Architectures: ResNet-20 and MobileNetV2 on 32x32 inputs (paper,
Implementation), the HeavyEarlyResNet20 / PlainConvNet20 variants (paper,
Analysis of Initial Hypotheses) and a 1-block-per-stage ResNet-8 used as the
small test case.  Only shapes live here; no arithmetic of the method.
"""
from __future__ import annotations

import numpy as np

DESC_FIELDS = ("kind", "cin", "cout", "kh", "kw", "stride", "pad", "hin", "win",
               "input", "residual", "act", "scheme_slot")
KIND_CONV, KIND_DEPTHWISE, KIND_FC = 0, 1, 2
ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2


def _node(kind, cin, cout, k, stride, hin, inp, residual=-1, act=ACT_NONE, slot=-1, name=""):
    pad = 1 if k == 3 else 0
    return dict(kind=kind, cin=cin, cout=cout, kh=k, kw=k, stride=stride, pad=pad,
                hin=hin, win=hin, input=inp, residual=residual, act=act,
                scheme_slot=slot, name=name)


def _hout(n):
    return (n["hin"] + 2 * n["pad"] - n["kh"]) // n["stride"] + 1


def resnet_cifar(blocks_per_stage=3, widths=(16, 32, 64), stem_width=None, n_classes=10, hin=32):
    """CIFAR-style ResNet with basic blocks: ResNet-20 for blocks_per_stage=3.

    ``widths`` gives the channel count of each stage; a stage whose width or
    resolution differs from its input starts with a strided block whose
    shortcut is a 1x1 projection (FP32-only, not a scheme layer).
    """
    nodes = []
    slot = 0
    stem_width = widths[0] if stem_width is None else stem_width
    nodes.append(_node(KIND_CONV, 3, stem_width, 3, 1, hin, -1, act=ACT_RELU, slot=slot, name="stem"))
    slot += 1
    prev, cin, h = 0, stem_width, hin
    for si, width in enumerate(widths):
        for bi in range(blocks_per_stage):
            stride = 2 if (si > 0 and bi == 0) else 1
            c1 = len(nodes)
            nodes.append(_node(KIND_CONV, cin, width, 3, stride, h, prev, act=ACT_RELU, slot=slot,
                               name=f"s{si + 1}b{bi}c1"))
            slot += 1
            if stride != 1 or cin != width:
                res = len(nodes)
                nodes.append(_node(KIND_CONV, cin, width, 1, stride, h, prev, act=ACT_NONE, slot=-1,
                                   name=f"s{si + 1}b{bi}sc"))
            else:
                res = prev
            h2 = _hout(nodes[c1])
            c2 = len(nodes)
            nodes.append(_node(KIND_CONV, width, width, 3, 1, h2, c1, residual=res, act=ACT_RELU,
                               slot=slot, name=f"s{si + 1}b{bi}c2"))
            slot += 1
            prev, cin, h = c2, width, h2
    nodes.append(_node(KIND_FC, cin, n_classes, 1, 1, h, prev, act=ACT_NONE, slot=slot, name="fc"))
    return nodes


def heavy_early_resnet20():
    """ResNet-20 with the channel progression reversed: stem 64, stages 32/16/16."""
    return resnet_cifar(3, widths=(32, 16, 16), stem_width=64)


def plain_convnet20(width=64, n_classes=10, hin=32):
    """20 plain 3x3 convolutions of equal width, then the classifier (21 scheme layers).

    The paper does not give the resolution schedule; stride 2 is placed at
    layers 7 and 14 so that the spatial sizes follow ResNet-20's 32/16/8.
    """
    nodes = []
    h, cin, prev = hin, 3, -1
    for i in range(20):
        stride = 2 if i in (7, 14) else 1
        nodes.append(_node(KIND_CONV, cin, width, 3, stride, h, prev, act=ACT_RELU, slot=i, name=f"f{3 * i}"))
        h = _hout(nodes[-1])
        cin, prev = width, i
    nodes.append(_node(KIND_FC, cin, n_classes, 1, 1, h, prev, act=ACT_NONE, slot=20, name="cls"))
    return nodes


def mobilenetv2_32(n_classes=10, hin=32):
    """MobileNetV2 (width 1.0) for 32x32 inputs, 53 scheme layers.

    Stem stride 1 and the first two stride-2 stages kept at stride 1, so the
    resolution schedule is 32 -> 16 -> 8.
    """
    cfg = [(1, 16, 1, 1), (6, 24, 2, 1), (6, 32, 3, 1), (6, 64, 4, 2),
           (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]
    nodes = []
    slot = 0
    nodes.append(_node(KIND_CONV, 3, 32, 3, 1, hin, -1, act=ACT_RELU6, slot=slot, name="stem"))
    slot += 1
    prev, cin, h = 0, 32, hin
    bidx = 0
    for t, c, n, s in cfg:
        for i in range(n):
            stride = s if i == 0 else 1
            hidden = cin * t
            x_in = prev
            cur = prev
            if t != 1:
                nodes.append(_node(KIND_CONV, cin, hidden, 1, 1, h, cur, act=ACT_RELU6, slot=slot,
                                   name=f"b{bidx}expand"))
                slot += 1
                cur = len(nodes) - 1
            nodes.append(_node(KIND_DEPTHWISE, hidden, hidden, 3, stride, h, cur, act=ACT_RELU6, slot=slot,
                               name=f"b{bidx}dw"))
            slot += 1
            cur = len(nodes) - 1
            h2 = _hout(nodes[cur])
            res = x_in if (stride == 1 and cin == c) else -1
            nodes.append(_node(KIND_CONV, hidden, c, 1, 1, h2, cur, residual=res, act=ACT_NONE, slot=slot,
                               name=f"b{bidx}project"))
            slot += 1
            prev, cin, h = len(nodes) - 1, c, h2
            bidx += 1
    nodes.append(_node(KIND_CONV, cin, 1280, 1, 1, h, prev, act=ACT_RELU6, slot=slot, name="last"))
    slot += 1
    prev = len(nodes) - 1
    nodes.append(_node(KIND_FC, 1280, n_classes, 1, 1, h, prev, act=ACT_NONE, slot=slot, name="fc"))
    return nodes


def desc_array(nodes):
    """int32 array [n_nodes][13] in DESC_FIELDS order (the C boundary's record)."""
    return np.array([[n[f] for f in DESC_FIELDS] for n in nodes], dtype=np.int32)


def n_scheme_layers(nodes):
    return 1 + max(n["scheme_slot"] for n in nodes)
