"""Shapes of the MobileNetV2 (width 1.0, 224x224) layers the path is measured on.

The bottleneck table (t, c, n, s) is the public MobileNetV2 architecture:
stem 3x3 s2 -> 32, then (1,16,1,1) (6,24,2,2) (6,32,3,2) (6,64,4,2) (6,96,3,1)
(6,160,3,2) (6,320,1,1), then a 1x1 conv to 1280 and a 1000-way classifier.
A block with t == 1 has no expansion conv, so the network has
1 + 16*2 + 1 = 34 pointwise convolutions and 17 depthwise ones.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List

BOTTLENECKS = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2),
               (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]
STEM_CHANNELS = 32
HEAD_CHANNELS = 1280
NUM_CLASSES = 1000
INPUT_RES = 224


@dataclass(frozen=True)
class PwShape:
    name: str
    hw: int        # spatial size H = W of input and output
    cin: int
    cout: int
    residual: bool  # a stride-1, cin==cout block adds its input after this projection


@dataclass(frozen=True)
class DwShape:
    name: str
    hw_in: int
    c: int
    stride: int


@dataclass(frozen=True)
class BlockShape:
    name: str
    hw_in: int
    cin: int
    t: int       # expansion factor; 1 = no expansion convolution
    cout: int
    stride: int


def mobilenetv2_blocks(input_hw: int = INPUT_RES // 2) -> List[BlockShape]:
    """The 17 inverted-residual blocks in network order; input_hw is the spatial size after the
    stem (112 for 224x224 images; smaller values give the same chain on smaller maps)."""
    out: List[BlockShape] = []
    hw, cin, b = input_hw, STEM_CHANNELS, 0
    for t, c, n, s in BOTTLENECKS:
        for i in range(n):
            b += 1
            stride = s if i == 0 else 1
            out.append(BlockShape(f"b{b}", hw, cin, t, c, stride))
            hw, cin = (hw + 2 - 3) // stride + 1, c
    return out


def _walk():
    pw: List[PwShape] = []
    dw: List[DwShape] = []
    hw = INPUT_RES // 2  # after the stride-2 stem
    cin = STEM_CHANNELS
    b = 0
    for t, c, n, s in BOTTLENECKS:
        for i in range(n):
            b += 1
            stride = s if i == 0 else 1
            hidden = cin * t
            if t != 1:
                pw.append(PwShape(f"b{b}.expand", hw, cin, hidden, False))
            dw.append(DwShape(f"b{b}.dw", hw, hidden, stride))
            hw_out = (hw + 2 - 3) // stride + 1
            pw.append(PwShape(f"b{b}.project", hw_out, hidden, c,
                              stride == 1 and cin == c))
            hw, cin = hw_out, c
    pw.append(PwShape("head.1x1", hw, cin, HEAD_CHANNELS, False))
    return pw, dw


def mobilenetv2_pointwise_layers() -> List[PwShape]:
    return _walk()[0]


def mobilenetv2_depthwise_layers() -> List[DwShape]:
    return _walk()[1]


def mobilenetv2_param_counts() -> Dict[str, int]:
    """Weight counts by layer kind (no biases except the classifier's, BatchNorm
    affine pairs counted separately), for checking the enumeration against the
    parameter shares the paper states."""
    pw, dw = _walk()
    n_pw = sum(p.cin * p.cout for p in pw)
    n_dw = sum(9 * d.c for d in dw)
    stem = 3 * 3 * 3 * STEM_CHANNELS
    fc = HEAD_CHANNELS * NUM_CLASSES + NUM_CLASSES
    bn_channels = STEM_CHANNELS + sum(p.cout for p in pw) + sum(d.c for d in dw)
    return {"pointwise": n_pw, "depthwise": n_dw, "stem": stem, "classifier": fc,
            "batchnorm_affine": 2 * bn_channels}


# The five measurement / parity configurations (shapes only; distributions are the
# generator defaults unless noted).
BASELINE_CONFIGS = {
    0: dict(kind="pw", n=1, h=14, w=14, cin=64, cout=384, act_window=(0, 127), residual=False),
    1: dict(kind="pw", n=32, h=56, w=56, cin=24, cout=144, act_window=(0, 127), residual=False),
    2: dict(kind="pw", n=256, h=7, w=7, cin=960, cout=160, act_window=(-128, 127), residual=True),
    3: dict(kind="sweep", n=128),
    4: dict(kind="block", n=64, h=28, w=28, cin=32, t=6, stride=1),
}
