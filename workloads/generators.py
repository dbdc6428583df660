"""Counter-based seeded generators for every tensor the path consumes.

Recipe (all integer draws, both ends inclusive):
  activations x     int8  NHWC, uniform in [0, 127]        (or full signed range on request)
  ternary weights   int8  [Cout][Cin], P(-1)=P(+1)=1/4, P(0)=1/2 by default;
                    a different zero fraction can be requested (P(+1)=P(-1))
  bias              int32 uniform in [-2^12, 2^12]
  multiplier        int32 uniform in [2^30, 2^31 - 1]
  shift             int32 uniform in [8, 14]
  residual          int8  uniform in [-64, 63]
  depthwise weights int8  [3][3][C], uniform in [-127, 127]

The generator is SplitMix64 used as a counter-based generator: draw i of a
stream is mix(seed + (i+1)*GOLDEN), so any slice of a tensor can be produced
independently and the values do not depend on chunking.  Each tensor of a
layer has its own stream, derived from (base seed, layer tag, tensor tag).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

CONFIG_SEED_BASE = 0x50524F4D  # "PROM"

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


class SplitMix64:
    """Counter-based stream of 64-bit words: word(i) = mix(seed + (i+1)*GOLDEN)."""

    def __init__(self, seed: int):
        self.seed = np.uint64(seed & 0xFFFFFFFFFFFFFFFF)

    def words(self, start: int, count: int) -> np.ndarray:
        with np.errstate(over="ignore"):
            idx = np.arange(start + 1, start + 1 + count, dtype=np.uint64)
            return _mix(self.seed + idx * _GOLDEN)

    def substream(self, tag: int) -> "SplitMix64":
        with np.errstate(over="ignore"):
            s = _mix(np.array([self.seed ^ (np.uint64(tag & 0xFFFFFFFFFFFFFFFF) * _M2)],
                              dtype=np.uint64))[0]
        return SplitMix64(int(s))

    # -- typed draws -------------------------------------------------------
    def bytes_masked(self, count: int, mask: int, chunk: int = 1 << 22) -> np.ndarray:
        """count bytes, each = (one byte of the word stream) & mask. 8 bytes per word,
        little-endian order inside the word."""
        out = np.empty(count, dtype=np.uint8)
        nwords = (count + 7) // 8
        pos = 0
        for w0 in range(0, nwords, chunk):
            n = min(chunk, nwords - w0)
            b = self.words(w0, n).view(np.uint8)  # little-endian host
            take = min(b.size, count - pos)
            out[pos:pos + take] = b[:take]
            pos += take
        if mask != 0xFF:
            np.bitwise_and(out, np.uint8(mask), out=out)
        return out

    def uniform_int(self, count: int, lo: int, hi: int) -> np.ndarray:
        """count integers uniform in [lo, hi] (inclusive) by multiply-shift on the
        high 32 bits of each word: lo + ((w >> 32) * span >> 32)."""
        span = np.uint64(hi - lo + 1)
        w = self.words(0, count) >> np.uint64(32)
        return (lo + ((w * span) >> np.uint64(32)).astype(np.int64))


def _ternary(stream: SplitMix64, count: int, p_zero: float) -> np.ndarray:
    """Ternary values with P(0)=p_zero and P(+1)=P(-1)=(1-p_zero)/2.
    One byte u of the stream per weight: u < T0 -> 0; else sign = lowest bit of the
    remaining range split in two halves."""
    u = stream.bytes_masked(count, 0xFF).astype(np.int32)
    t0 = int(round(p_zero * 256.0))
    half = (256 - t0) // 2
    w = np.zeros(count, dtype=np.int8)
    w[(u >= t0) & (u < t0 + half)] = 1
    w[u >= t0 + half] = -1
    if (256 - t0) % 2:  # odd remainder: give the last code to zero to keep +/- balanced
        w[u == 255] = 0
    return w


@dataclass
class PwLayerInputs:
    n: int
    h: int
    w: int
    cin: int
    cout: int
    x: np.ndarray            # int8 [n,h,w,cin]
    weight: np.ndarray       # int8 [cout,cin] in {-1,0,1}
    bias: np.ndarray         # int32 [cout]
    mult: np.ndarray         # int32 [cout]
    shift: np.ndarray        # int32 [cout]
    act_min: int
    act_max: int
    residual: Optional[np.ndarray]  # int8 [n,h,w,cout] or None

    @property
    def m(self) -> int:
        return self.n * self.h * self.w


@dataclass
class DwLayerInputs:
    n: int
    h: int
    w: int
    c: int
    stride: int
    x: np.ndarray            # int8 [n,h,w,c]
    weight: np.ndarray       # int8 [3,3,c]
    bias: np.ndarray
    mult: np.ndarray
    shift: np.ndarray
    act_min: int
    act_max: int


@dataclass
class BlockInputs:
    n: int
    h: int
    w: int
    cin: int
    chid: int
    cout: int
    stride: int
    add_residual: bool
    x: np.ndarray
    expand: PwLayerInputs     # x field unused (shares block x)
    dw: DwLayerInputs         # x field unused
    project: PwLayerInputs    # x field unused


def _requant_params(stream: SplitMix64, c: int, shift_range: Tuple[int, int] = (8, 14)):
    bias = stream.substream(11).uniform_int(c, -(1 << 12), 1 << 12).astype(np.int32)
    mult = stream.substream(12).uniform_int(c, 1 << 30, (1 << 31) - 1).astype(np.int32)
    shift = stream.substream(13).uniform_int(c, shift_range[0], shift_range[1]).astype(np.int32)
    return bias, mult, shift


def prelu_mult_neg(seed: int, mult: np.ndarray) -> np.ndarray:
    """Negative-side multipliers of a PReLU layer: slope a_c = k/256 with k uniform in
    [-64, 255] (PReLU slopes start at 0.25 and are learned per channel; a few turn negative),
    folded into the positive multiplier, mult_neg = floor(mult * k / 256).  Input recipe only:
    the layer functions take mult_neg as given."""
    k = SplitMix64(seed).substream(31).uniform_int(mult.size, -64, 255).astype(np.int64)
    return ((mult.astype(np.int64) * k) >> 8).astype(np.int32)


def make_pw_layer(seed: int, n: int, h: int, w: int, cin: int, cout: int, *,
                  act_window: Tuple[int, int] = (0, 127), with_residual: bool = False,
                  p_zero: float = 0.5, signed_x: bool = False,
                  shift_range: Tuple[int, int] = (8, 14), make_x: bool = True) -> PwLayerInputs:
    """All tensors of one ternary pointwise layer, from one seed."""
    root = SplitMix64(seed)
    m = n * h * w
    if make_x:
        if signed_x:
            x = root.substream(1).bytes_masked(m * cin, 0xFF).view(np.int8)
        else:
            x = root.substream(1).bytes_masked(m * cin, 0x7F).view(np.int8)
        x = x.reshape(n, h, w, cin)
    else:
        x = np.empty((0,), dtype=np.int8)
    weight = _ternary(root.substream(2), cout * cin, p_zero).reshape(cout, cin)
    bias, mult, shift = _requant_params(root.substream(3), cout, shift_range)
    residual = None
    if with_residual:
        r = root.substream(4).bytes_masked(m * cout, 0x7F).astype(np.int16) - 64
        residual = r.astype(np.int8).reshape(n, h, w, cout)
    return PwLayerInputs(n, h, w, cin, cout, x, weight, bias, mult, shift,
                         act_window[0], act_window[1], residual)


def make_dw_layer(seed: int, n: int, h: int, w: int, c: int, stride: int = 1, *,
                  act_window: Tuple[int, int] = (0, 127), signed_x: bool = False,
                  shift_range: Tuple[int, int] = (8, 14), make_x: bool = True) -> DwLayerInputs:
    root = SplitMix64(seed)
    if make_x:
        mask = 0xFF if signed_x else 0x7F
        x = root.substream(1).bytes_masked(n * h * w * c, mask).view(np.int8).reshape(n, h, w, c)
    else:
        x = np.empty((0,), dtype=np.int8)
    weight = root.substream(2).uniform_int(9 * c, -127, 127).astype(np.int8).reshape(3, 3, c)
    bias, mult, shift = _requant_params(root.substream(3), c, shift_range)
    return DwLayerInputs(n, h, w, c, stride, x, weight, bias, mult, shift,
                         act_window[0], act_window[1])


@dataclass
class GconvLayerInputs:
    n: int
    h: int
    w: int
    c: int
    gs: int
    stride: int
    x: np.ndarray            # int8 [n,h,w,c]
    weight: np.ndarray       # int8 [3,3,c,gs]
    bias: np.ndarray
    mult: np.ndarray
    shift: np.ndarray
    act_min: int
    act_max: int


def make_gconv_layer(seed: int, n: int, h: int, w: int, c: int, gs: int, stride: int = 1, *,
                     act_window: Tuple[int, int] = (0, 127), signed_x: bool = False,
                     shift_range: Tuple[int, int] = (10, 16), make_x: bool = True) -> GconvLayerInputs:
    """A grouped 3x3 layer (groups of gs channels, as many outputs as inputs): 8-bit weights
    uniform in [-127, 127] like the depthwise layers."""
    root = SplitMix64(seed)
    if make_x:
        mask = 0xFF if signed_x else 0x7F
        x = root.substream(1).bytes_masked(n * h * w * c, mask).view(np.int8).reshape(n, h, w, c)
    else:
        x = np.empty((0,), dtype=np.int8)
    weight = root.substream(2).uniform_int(9 * c * gs, -127, 127).astype(np.int8).reshape(3, 3, c, gs)
    bias, mult, shift = _requant_params(root.substream(3), c, shift_range)
    return GconvLayerInputs(n, h, w, c, gs, stride, x, weight, bias, mult, shift,
                            act_window[0], act_window[1])


def make_block(seed: int, n: int, h: int, w: int, cin: int, t: int, cout: Optional[int] = None,
               stride: int = 1, *, signed_x: bool = False, p_zero: float = 0.5,
               expand_shift: Tuple[int, int] = (8, 14), dw_shift: Tuple[int, int] = (8, 14),
               project_shift: Tuple[int, int] = (8, 14)) -> BlockInputs:
    """Inverted-residual block: expand (clamp [0,127]) -> depthwise 3x3 (clamp [0,127]) ->
    project (clamp [-128,127]) + saturating add of the block input when stride==1 and
    cin==cout."""
    cout = cin if cout is None else cout
    chid = cin * t
    root = SplitMix64(seed)
    mask = 0xFF if signed_x else 0x7F
    x = root.substream(1).bytes_masked(n * h * w * cin, mask).view(np.int8).reshape(n, h, w, cin)
    ho = (h + 2 - 3) // stride + 1
    wo = (w + 2 - 3) // stride + 1
    expand = make_pw_layer(int(root.substream(21).seed), n, h, w, cin, chid,
                           act_window=(0, 127), p_zero=p_zero, shift_range=expand_shift, make_x=False)
    dw = make_dw_layer(int(root.substream(22).seed), n, h, w, chid, stride,
                       act_window=(0, 127), shift_range=dw_shift, make_x=False)
    project = make_pw_layer(int(root.substream(23).seed), n, ho, wo, chid, cout,
                            act_window=(-128, 127), p_zero=p_zero, shift_range=project_shift, make_x=False)
    add_res = (stride == 1 and cin == cout)
    return BlockInputs(n, h, w, cin, chid, cout, stride, add_res, x, expand, dw, project)


def float_conv_weights(seed: int, cout: int, fan: int, *, kind: str = "kaiming") -> np.ndarray:
    """Seeded float32 weights [cout][fan] as a network holds them before quantisation: Kaiming
    normal (std sqrt(2/cout), the initialisation the paper's appendix analyses) or, with
    kind="trained", the same with every tenth row scaled by 1e-3 .. 1e3 and a few exact zeros and
    half-way values planted, to exercise the per-channel scale, the eps clamp and the rounding ties."""
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((cout, fan)) * np.sqrt(2.0 / cout)).astype(np.float32)
    if kind == "trained":
        for i in range(0, cout, 10):
            w[i] *= np.float32(10.0 ** rng.integers(-3, 4))
        w[rng.integers(0, cout, 8), rng.integers(0, fan, 8)] = 0.0
        if cout > 3:
            w[3] = 0.0            # a dead channel: the eps clamp decides
        if cout > 5 and fan >= 4:
            w[5, :] = 0.0
            w[5, :4] = np.array([0.5, -0.5, 1.5, -1.5], dtype=np.float32)[: min(4, fan)]
    return w
