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
