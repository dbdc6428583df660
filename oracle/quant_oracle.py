"""CPU oracle of the weight quantisers that feed the path (test infrastructure only; the HIP
product path never imports this).

What it computes follows the paper's Section 3.1 and its pseudocode of the weight quantisation
(appendix figure "quantization of conv weights"), where the two disagree the pseudocode:
  pointwise (ternary, channel-wise absmean)
      scale_i = 1 / max(mean_j |W[i][j]|, eps)             (the pseudocode clamps the mean at eps;
                                                            Eq. 3 adds eps instead)
      What[i][j] = clamp(round(W[i][j] * scale_i), -1, 1)
  depthwise (8-bit, channel-wise absmax)
      scale_i = 127 / max(max_{k,l} |W[i][k][l]|, eps)      (the pseudocode has the factor 127 that
                                                            Eq. 5 leaves out)
      What[i][k][l] = clamp(round(W * scale_i), -128, 127)
round() is round-half-to-even, as torch.round in the pseudocode.

Precision.  The paper's code runs in float32 and a quantised code is decided by a float32
product, so the decision is taken in float32 here as well: the mean of |W| is the sum of the row
in float64 (sequential, numpy's) divided by cin and rounded once to float32 -- the one place where
the order of a float32 reduction would otherwise be left to the implementation --, the scale is
one correctly rounded float32 division, and W * scale is one float32 multiplication.
"""
from __future__ import annotations

import numpy as np


def quantize_pw_absmean(w: np.ndarray, eps: float = 1e-5):
    """w: float32 [cout][cin].  Returns (codes int8 [cout][cin] in {-1,0,1}, scale float32 [cout])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    cout, cin = w.shape
    mean = np.empty(cout, dtype=np.float32)
    for i in range(cout):
        s = 0.0
        for v in np.abs(w[i]).astype(np.float64):  # plain sequential float64 sum
            s += float(v)
        mean[i] = np.float32(s / cin)
    scale = (np.float32(1.0) / np.maximum(mean, np.float32(eps))).astype(np.float32)
    q = np.rint((w * scale[:, None]).astype(np.float32))  # float32 product, half-to-even
    return np.clip(q, -1, 1).astype(np.int8), scale


def quantize_dw_absmax(w: np.ndarray, eps: float = 1e-5):
    """w: float32 [c][3][3] (one 3x3 filter per channel, the paper's [c_out,1,k,k] without the
    singleton).  Returns (q int8 [3][3][c], the layout prom_dw_conv takes, scale float32 [c])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    c = w.shape[0]
    amax = np.max(np.abs(w.reshape(c, -1)), axis=1).astype(np.float32)
    scale = (np.float32(127.0) / np.maximum(amax, np.float32(eps))).astype(np.float32)
    q = np.rint((w.reshape(c, -1) * scale[:, None]).astype(np.float32))
    q = np.clip(q, -128, 127).astype(np.int8).reshape(c, 3, 3)
    return np.ascontiguousarray(np.transpose(q, (1, 2, 0))), scale


def quantize_gconv_absmax(w: np.ndarray, eps: float = 1e-5):
    """The same absmax scheme (Section 3.1, Eq. 4-5 with the factor 127 and the eps clamp of the
    pseudocode) for a grouped 3x3 layer: one scale per output channel over its group's input
    channels and the 9 taps.  w: float32 [c][gs][3][3] (the paper's [c_out][c_in per group][k][k]).
    Returns (q int8 [3][3][c][gs], the layout prom_gconv3x3 takes, scale float32 [c])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    c, gs = w.shape[0], w.shape[1]
    assert w.shape[2:] == (3, 3)
    amax = np.max(np.abs(w.reshape(c, -1)), axis=1).astype(np.float32)
    scale = (np.float32(127.0) / np.maximum(amax, np.float32(eps))).astype(np.float32)
    q = np.rint((w.reshape(c, -1) * scale[:, None]).astype(np.float32))
    q = np.clip(q, -128, 127).astype(np.int8).reshape(c, gs, 3, 3)
    return np.ascontiguousarray(np.transpose(q, (2, 3, 0, 1))), scale


def quantize_activation_absmax(x: np.ndarray, eps: float = 1e-5):
    """The paper's activation quantiser (Section 3.1, Eq. 6-7, with the factor 127 and the eps
    clamp of its pseudocode): one scale per batch element over all its channels and pixels.
    x: float32 [n][...].  Returns (q int8, same shape; scale float32 [n]).  The maximum is exact,
    the scale one float32 division, the code one float32 product rounded half to even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    n = x.shape[0]
    flat = x.reshape(n, -1)
    amax = np.max(np.abs(flat), axis=1).astype(np.float32)
    scale = (np.float32(127.0) / np.maximum(amax, np.float32(eps))).astype(np.float32)
    q = np.rint((flat * scale[:, None]).astype(np.float32))
    return np.clip(q, -128, 127).astype(np.int8).reshape(x.shape), scale
