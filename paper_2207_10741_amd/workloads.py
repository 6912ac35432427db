"""Layer lists of the benchmark workloads (shapes only, no arithmetic).

The paper evaluates on whole detection networks with pretrained weights
(Sec. III-B); those are not available, so conv stacks with the shapes of
well-known classification backbones stand in.  A stack is a list of `Op`s; each
reads the output of an earlier op (`src`, -1 = the stack's input) so that the
1x1 projection convs of residual networks can consume their block's input.
There are no batch-norms and no residual adds: every conv is followed by ReLU.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List


@dataclass(frozen=True)
class Op:
    kind: str      # "conv", "dwconv" (one filter per channel; c_out == c_in) or "maxpool"
    name: str
    c_in: int
    c_out: int
    k: int
    stride: int
    pad: int
    src: int       # index of the op whose output is read; -1 = stack input
    relu: bool = True


def resnet18() -> List[Op]:
    """All 20 convs of ResNet-18 (7x7/2 stem, 16 3x3, three 1x1/2 projections)
    and the 3x3/2 stem max-pool."""
    ops: List[Op] = [Op("conv", "conv1", 3, 64, 7, 2, 3, -1), Op("maxpool", "pool1", 64, 64, 3, 2, 1, 0)]
    c_prev = 64
    last = 1
    for stage, c in enumerate((64, 128, 256, 512), start=1):
        for blk in range(2):
            block_in = last
            s = 2 if (stage > 1 and blk == 0) else 1
            ops.append(Op("conv", "s%db%d_a" % (stage, blk), c_prev, c, 3, s, 1, block_in))
            ops.append(Op("conv", "s%db%d_b" % (stage, blk), c, c, 3, 1, 1, len(ops) - 1))
            last = len(ops) - 1
            if s == 2:
                ops.append(Op("conv", "s%db%d_down" % (stage, blk), c_prev, c, 1, 2, 0, block_in))
            c_prev = c
    return ops


def resnet50_bottlenecks() -> List[Op]:
    """The 52 convs of ResNet-50's 16 bottleneck blocks (1x1 / 3x3 / 1x1, plus a
    1x1 projection on the first block of each stage).  Stride 2 sits on the 3x3
    of the first block of stages 2-4.  Input: the post-stem activation, 64
    channels at 1/4 of the image side."""
    ops: List[Op] = []
    c_prev = 64
    last = -1
    for stage, (mid, blocks) in enumerate(((64, 3), (128, 4), (256, 6), (512, 3)), start=1):
        c_out = 4 * mid
        for blk in range(blocks):
            block_in = last
            s = 2 if (stage > 1 and blk == 0) else 1
            ops.append(Op("conv", "s%db%d_1x1a" % (stage, blk), c_prev, mid, 1, 1, 0, block_in))
            ops.append(Op("conv", "s%db%d_3x3" % (stage, blk), mid, mid, 3, s, 1, len(ops) - 1))
            ops.append(Op("conv", "s%db%d_1x1b" % (stage, blk), mid, c_out, 1, 1, 0, len(ops) - 1))
            last = len(ops) - 1
            if blk == 0:
                ops.append(Op("conv", "s%db%d_down" % (stage, blk), c_prev, c_out, 1, s, 0, block_in))
            c_prev = c_out
    return ops


def vgg16() -> List[Op]:
    """VGG-16's 13 3x3 convs with 2x2/2 max-pools after convs 2, 4, 7 and 10."""
    ops: List[Op] = []
    c_prev = 3
    i = 0
    for c, reps in ((64, 2), (128, 2), (256, 3), (512, 3), (512, 3)):
        for _ in range(reps):
            i += 1
            ops.append(Op("conv", "conv%d" % i, c_prev, c, 3, 1, 1, len(ops) - 1))
            c_prev = c
        if i < 13:
            ops.append(Op("maxpool", "pool%d" % i, c, c, 2, 2, 0, len(ops) - 1))
    return ops


def mobilenetv2() -> List[Op]:
    """The 52 convs of a MobileNetV2 backbone (SSD-Lite's backbone, Sec. IV): 3x3/2 stem, 17
    inverted-residual blocks (1x1 expansion - none in the first block -, 3x3 depthwise, 1x1
    projection), the final 1x1.  No residual adds; like the other stacks every conv is followed
    by ReLU, the projections too, which keeps magnitudes steady under He-normal weights."""
    ops: List[Op] = [Op("conv", "stem", 3, 32, 3, 2, 1, -1)]
    c_prev = 32
    settings = ((1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2),
                (6, 320, 1, 1))
    for bi, (t, c, reps, s) in enumerate(settings):
        for r in range(reps):
            mid = c_prev * t
            if t != 1:
                ops.append(Op("conv", "b%dr%d_expand" % (bi, r), c_prev, mid, 1, 1, 0, len(ops) - 1))
            ops.append(Op("dwconv", "b%dr%d_dw" % (bi, r), mid, mid, 3, s if r == 0 else 1, 1, len(ops) - 1))
            ops.append(Op("conv", "b%dr%d_project" % (bi, r), mid, c, 1, 1, 0, len(ops) - 1))
            c_prev = c
    ops.append(Op("conv", "head", c_prev, 1280, 1, 1, 0, len(ops) - 1))
    return ops


def sweep_shapes():
    """(C, side) of ResNet-50's four 3x3 layer shapes for a 512x512 image."""
    return [(64, 128), (128, 64), (256, 32), (512, 16)]


def mobilenetv2_depthwise():
    """(channels, input side, stride) of the 3x3 depthwise layers of a MobileNetV2 backbone (the
    backbone of SSD-Lite, Sec. IV) on 224 x 224 images; repeats of a shape listed once."""
    return [(32, 112, 1), (96, 112, 2), (144, 56, 1), (144, 56, 2), (192, 28, 1), (192, 28, 2),
            (384, 14, 1), (576, 14, 1), (576, 14, 2), (960, 7, 1)]


def resnet50_pointwise():
    """(input channels, output channels, divisor of the post-stem side) of 1x1 layers of a ResNet-50
    with up to 512 input channels: the reductions and expansions of the four stages' bottlenecks
    (repeats of a shape listed once, projections with a stride left out)."""
    return [(64, 64, 1), (64, 256, 1), (256, 64, 1), (256, 128, 1),
            (128, 512, 2), (512, 128, 2), (512, 256, 2),
            (256, 1024, 4), (512, 2048, 8)]


def mobilenetv2_pointwise():
    """(input channels, output channels, divisor of the image side) of the 1x1 layers of a MobileNetV2
    backbone (the expansions and projections of its inverted-residual blocks and the final layer);
    repeats of a shape listed once."""
    return [(32, 16, 2), (16, 96, 2), (96, 24, 4), (24, 144, 4), (144, 24, 4), (144, 32, 8), (32, 192, 8),
            (192, 32, 8), (192, 64, 16), (64, 384, 16), (384, 64, 16), (384, 96, 16), (96, 576, 16),
            (576, 96, 16), (576, 160, 32), (160, 960, 32), (960, 160, 32), (960, 320, 32), (320, 1280, 32)]


POINTWISE_BATCH, POINTWISE_H, POINTWISE_W = 32, 120, 160   # the post-stem activation of 480 x 640 images
DEPTHWISE_BATCH = 32
SWEEP_BATCH = 16
HEADLINE_IRRELEVANT = 0.48   # Sec. II-B: the paper's overall irrelevant-pixel share
