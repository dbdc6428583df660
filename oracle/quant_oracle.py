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


def pw_conv_dynamic_quant(x, weight, x_step, w_scale, bias=None, relu: bool = False, eps: float = 1e-5):
    """A ternary pointwise layer followed by the paper's activation quantiser (Section 3.1:
    Eq. 1-3 give the weight scale, Eq. 6-7 the per-image activation scale, with the factor 127 and
    the eps clamp of the pseudocode), from integer inputs to integer outputs:

        acc[m][co] = sum_k x[m][k] * weight[co][k]                    (exact integers)
        z[m][co]   = (float(acc) * w_scale[co]) * x_step[i] + bias[co]  i = image of pixel m;
                     each of the three operations rounded once to float32, in this order
        z          = max(z, 0) if relu
        amax[i]    = max over the image's pixels and channels |z|
        scale[i]   = 127 / max(amax[i], eps)                           (one float32 division)
        q[m][co]   = clamp(round_half_even(z * scale[i]), -128, 127)   (one float32 product)

    x int8 [n][h][w][cin] with real value x * x_step[i] (x_step = amax_in / 127, the reciprocal
    of the scale the quantiser of the previous layer returned); weight int8 [cout][cin] in
    {-1,0,1} with real value weight * w_scale[co] (w_scale = the absmean of Eq. 1);
    bias float32 [cout] or None (a folded normalisation shift).
    Returns (q int8 [n][h][w][cout], amax float32 [n], scale float32 [n]).
    Needs |acc| < 2^24 so that float(acc) is exact (cin <= 132104 for int8 activations)."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    weight = np.ascontiguousarray(weight, dtype=np.int8)
    n, h, w, cin = x.shape
    cout = weight.shape[0]
    assert weight.shape == (cout, cin) and 128 * cin < (1 << 24)
    x_step = np.asarray(x_step, dtype=np.float32).reshape(n)
    w_scale = np.asarray(w_scale, dtype=np.float32).reshape(cout)
    acc = x.reshape(n, h * w, cin).astype(np.int64) @ weight.T.astype(np.int64)      # [n][hw][cout]
    t = (acc.astype(np.float32) * w_scale[None, None, :]).astype(np.float32)
    z = (t * x_step[:, None, None]).astype(np.float32)
    if bias is not None:
        z = (z + np.asarray(bias, dtype=np.float32).reshape(1, 1, cout)).astype(np.float32)
    if relu:
        z = np.maximum(z, np.float32(0.0))
    amax = np.max(np.abs(z).reshape(n, -1), axis=1).astype(np.float32)
    scale = (np.float32(127.0) / np.maximum(amax, np.float32(eps))).astype(np.float32)
    q = np.rint((z * scale[:, None, None]).astype(np.float32))
    q = np.clip(q, -128, 127).astype(np.int8).reshape(n, h, w, cout)
    return q, amax, scale
