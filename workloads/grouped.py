"""Shapes of the grouped 3x3 convolutions of the other two architecture families the paper
evaluates (RegNetX and ResNeXt: Section 2 describes their group sizes above one, Section 5 lists
the models), from their public architecture tables at 224x224 input.  Each bottleneck block has
one grouped 3x3 conv with as many outputs as inputs; the first block of a stage has stride 2
(ResNeXt's first stage: stride 1)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List


@dataclass(frozen=True)
class GconvShape:
    name: str
    hw_in: int
    c: int
    gs: int
    stride: int


def _stages(prefix, hw, widths, depths, group_size_of, first_stride):
    out: List[GconvShape] = []
    for s, (wd, d) in enumerate(zip(widths, depths)):
        for b in range(d):
            stride = first_stride[s] if b == 0 else 1
            out.append(GconvShape(f"{prefix}.s{s + 1}.b{b + 1}", hw, wd, group_size_of(s, wd), stride))
            hw = (hw - 1) // stride + 1
    return out


def regnetx_400mf_grouped_layers() -> List[GconvShape]:
    """RegNetX-400MF: depths 1, 2, 7, 12; widths 32, 64, 160, 384; group width 16; the stem leaves
    112x112 and every stage starts with a stride-2 block."""
    return _stages("regnetx400", 112, (32, 64, 160, 384), (1, 2, 7, 12), lambda s, w: 16, (2, 2, 2, 2))


def resnext50_32x4d_grouped_layers() -> List[GconvShape]:
    """ResNeXt-50 32x4d: depths 3, 4, 6, 3; bottleneck widths 128, 256, 512, 1024 in 32 groups
    (group sizes 4, 8, 16, 32); 56x56 after the stem and the pooling."""
    return _stages("resnext50", 56, (128, 256, 512, 1024), (3, 4, 6, 3), lambda s, w: w // 32, (1, 2, 2, 2))


# ---- the pointwise (1x1) convolutions of the same two families ------------------------------------
# A bottleneck block is 1x1 (c_in -> width) at the block's input resolution, the grouped 3x3
# (which carries the stride), 1x1 (width -> c_out) at the output resolution, and, in the first
# block of a stage, a 1x1 shortcut (c_in -> c_out) that reads every stride-th pixel, i.e. works on
# the output resolution's pixel count.  The residual sum follows the last 1x1 of every block.
from .mobilenetv2 import PwShape  # noqa: E402


def _pointwise_of_stages(prefix, hw, c_in, widths, outs, depths, first_stride):
    out: List[PwShape] = []
    for s, (wd, co, d) in enumerate(zip(widths, outs, depths)):
        for b in range(d):
            stride = first_stride[s] if b == 0 else 1
            hw_out = (hw - 1) // stride + 1
            name = f"{prefix}.s{s + 1}.b{b + 1}"
            out.append(PwShape(name + ".reduce", hw, c_in, wd, False))
            if b == 0 and (stride != 1 or c_in != co):
                out.append(PwShape(name + ".shortcut", hw_out, c_in, co, False))
            out.append(PwShape(name + ".expand", hw_out, wd, co, True))
            hw, c_in = hw_out, co
    return out


def regnetx_400mf_pointwise_layers() -> List[PwShape]:
    """RegNetX-400MF (bottleneck ratio 1: width == c_out): 22 blocks, 48 pointwise convolutions,
    32 to 384 channels at 112x112 down to 7x7."""
    w = (32, 64, 160, 384)
    return _pointwise_of_stages("regnetx400", 112, 32, w, w, (1, 2, 7, 12), (2, 2, 2, 2))


def resnext50_32x4d_pointwise_layers() -> List[PwShape]:
    """ResNeXt-50 32x4d: 16 blocks, 36 pointwise convolutions, 64 to 2048 channels at 56x56 down
    to 7x7; the layers of the last two stages have more operations per byte than the int8 matrix
    units' balance point (2 K N / (K + N) > 5000 Top/s / 8 TB/s = 625)."""
    return _pointwise_of_stages("resnext50", 56, 64, (128, 256, 512, 1024), (256, 512, 1024, 2048),
                                (3, 4, 6, 3), (1, 2, 2, 2))
