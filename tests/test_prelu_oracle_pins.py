"""Pins of the oracle's PReLU requantisation (the paper's MobileNetV2 / RegNetX models use
PReLU where the original networks have ReLU6 / ReLU: Section 3.2, last paragraph).

The integer form is this build's contract; it is pinned here against
  - the plain requantisation, which it must equal when both multipliers are the same
    (slope 1) and, with the window raised to 0, when the negative multiplier is 0 (ReLU);
  - exact rational arithmetic with the multiplier picked by the sign of acc + bias;
  - torch's float64 PReLU on the dequantised pre-activation, within half a code;
  - hand-worked values.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from workloads import make_pw_layer, make_dw_layer, make_block, prelu_mult_neg


def test_hand_worked_values():
    # mult = 2^30, shift 0: positive side s/2; mult_neg = 2^28: negative side s/8; ties go up
    assert oracle.requant_prelu(1000, 1 << 30, 1 << 28, 0) == 500
    assert oracle.requant_prelu(-1000, 1 << 30, 1 << 28, 0) == -125
    assert oracle.requant_prelu(-4, 1 << 30, 1 << 28, 0) == 0       # -0.5 -> 0
    assert oracle.requant_prelu(-5, 1 << 30, 1 << 28, 0) == -1      # -0.625 -> -1
    assert oracle.requant_prelu(-12, 1 << 30, 1 << 28, 0) == -1     # -1.5 -> -1
    assert oracle.requant_prelu(0, 1 << 30, -(1 << 30), 0) == 0
    # a negative slope turns negative inputs positive
    assert oracle.requant_prelu(-1000, 1 << 30, -(1 << 29), 0) == 250
    assert oracle.requant_prelu(-1001, 1 << 30, -(1 << 29), 1) == 125   # 125.125
    assert oracle.requant_prelu(-1004, 1 << 30, -(1 << 29), 1) == 126   # 125.5 -> 126


def test_slope_one_is_the_plain_requantisation():
    rng = np.random.default_rng(7)
    for _ in range(20000):
        s = int(rng.integers(-(1 << 22), 1 << 22))
        mult = int(rng.integers(1 << 30, 1 << 31))
        shift = int(rng.integers(0, 32))
        assert oracle.requant_prelu(s, mult, mult, shift) == oracle.requant(s, mult, shift)


def test_slope_zero_is_relu():
    rng = np.random.default_rng(8)
    for _ in range(20000):
        s = int(rng.integers(-(1 << 22), 1 << 22))
        mult = int(rng.integers(1 << 30, 1 << 31))
        shift = int(rng.integers(0, 32))
        assert oracle.requant_prelu(s, mult, 0, shift) == max(oracle.requant(s, mult, shift), 0)


def test_exact_rationals_with_sign_selected_multiplier():
    rng = np.random.default_rng(9)
    for _ in range(20000):
        s = int(rng.integers(-(1 << 24), 1 << 24))
        mult = int(rng.integers(1, 1 << 31))
        mneg = int(rng.integers(-(1 << 31), 1 << 31))
        shift = int(rng.integers(0, 32))
        m = mult if s >= 0 else mneg
        want = math.floor(Fraction(s * m, 1 << (31 + shift)) + Fraction(1, 2))
        assert oracle.requant_prelu(s, mult, mneg, shift) == want
    for s in (-(1 << 30) - (1 << 23), (1 << 30) + (1 << 23), -1, 0, 1):
        for mneg in (-(1 << 31), (1 << 31) - 1, 0, 1, -1):
            for shift in (0, 1, 2, 31):
                m = ((1 << 31) - 1) if s >= 0 else mneg
                want = math.floor(Fraction(s * m, 1 << (31 + shift)) + Fraction(1, 2))
                assert oracle.requant_prelu(s, (1 << 31) - 1, mneg, shift) == want


def _float_prelu_codes(acc, bias, mult, mneg, shift, lo, hi):
    """torch's PReLU on z = s * sigma with sigma = mult / 2^(31+shift), slope = mneg/mult,
    in float64; returns z' (not rounded) so that the caller can bound the distance."""
    torch = pytest.importorskip("torch")
    s = acc.astype(np.int64) + bias.astype(np.int64)
    sigma = mult.astype(np.float64) / np.exp2(31.0 + shift.astype(np.float64))
    slope = mneg.astype(np.float64) / mult.astype(np.float64)
    z = torch.from_numpy(s.astype(np.float64) * sigma)                 # [..., C]
    zz = z.reshape(-1, z.shape[-1]).t().unsqueeze(0)                   # [1, C, M]: channel dim 1
    out = torch.nn.functional.prelu(zz, torch.from_numpy(slope))
    return out.squeeze(0).t().reshape(z.shape).numpy()


def test_pw_prelu_within_half_a_code_of_float_prelu():
    L = make_pw_layer(91, 2, 5, 7, 48, 40, signed_x=True, act_window=(-128, 127), shift_range=(2, 6))
    mneg = prelu_mult_neg(91, L.mult)
    assert (mneg < 0).any() and (mneg > 0).any()
    y = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -128, 127, mult_neg=mneg)
    acc = oracle.pw_accum(L.x, L.weight)
    f = _float_prelu_codes(acc, L.bias, L.mult, mneg, L.shift, -128, 127)
    inside = (f > -127.4) & (f < 126.4)
    assert inside.sum() > 0.5 * f.size
    assert np.all(np.abs(y[inside].astype(np.float64) - f[inside]) <= 0.5 + 1e-6)
    assert np.all(y[f >= 127] == 127) and np.all(y[f <= -128.5] == -128)
    # the sign decision uses acc + bias, not acc: there are outputs where the two differ
    s = acc.astype(np.int64) + L.bias
    assert ((s < 0) != (acc < 0)).any()


def test_dw_prelu_within_half_a_code_of_float_prelu():
    torch = pytest.importorskip("torch")
    D = make_dw_layer(92, 2, 6, 5, 12, 1, signed_x=True, act_window=(-128, 127), shift_range=(8, 10))
    mneg = prelu_mult_neg(92, D.mult)
    y = oracle.dw_conv(D.x, D.weight, 1, D.bias, D.mult, D.shift, -128, 127, mult_neg=mneg)
    xt = torch.from_numpy(D.x.astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(D.weight.astype(np.float64)).permute(2, 0, 1).unsqueeze(1)
    acc = torch.nn.functional.conv2d(xt, wt, padding=1, groups=12).permute(0, 2, 3, 1).numpy()
    f = _float_prelu_codes(np.rint(acc).astype(np.int64), D.bias, D.mult, mneg, D.shift, -128, 127)
    inside = (f > -127.4) & (f < 126.4)
    assert inside.sum() > 0.3 * f.size
    assert np.all(np.abs(y[inside].astype(np.float64) - f[inside]) <= 0.5 + 1e-6)


def test_layers_with_equal_multipliers_are_the_plain_layers():
    L = make_pw_layer(93, 1, 4, 6, 24, 20, signed_x=True, act_window=(-100, 90), with_residual=True)
    a = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -100, 90, residual=L.residual)
    b = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -100, 90, residual=L.residual,
                       mult_neg=L.mult)
    assert np.array_equal(a, b)
    D = make_dw_layer(94, 1, 7, 4, 9, 2, signed_x=True, act_window=(-128, 127))
    a = oracle.dw_conv(D.x, D.weight, 2, D.bias, D.mult, D.shift, -128, 127)
    b = oracle.dw_conv(D.x, D.weight, 2, D.bias, D.mult, D.shift, -128, 127, mult_neg=D.mult)
    assert np.array_equal(a, b)
    # slope 0 with the full window = the plain layer with the window cut at 0
    a = oracle.dw_conv(D.x, D.weight, 2, D.bias, D.mult, D.shift, 0, 127)
    b = oracle.dw_conv(D.x, D.weight, 2, D.bias, D.mult, D.shift, -128, 127,
                       mult_neg=np.zeros_like(D.mult))
    assert np.array_equal(a, b)


def test_residual_is_added_after_the_window():
    L = make_pw_layer(95, 1, 3, 3, 16, 8, signed_x=True, with_residual=True, shift_range=(2, 4))
    mneg = prelu_mult_neg(95, L.mult)
    plain = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -20, 20, mult_neg=mneg)
    withres = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -20, 20, mult_neg=mneg,
                             residual=L.residual)
    want = np.clip(plain.astype(np.int32) + L.residual, -128, 127).astype(np.int8)
    assert np.array_equal(withres, want)


def test_block_prelu_with_slope_one_windows_equals_plain_block():
    B = make_block(96, 1, 6, 6, 8, 3, stride=1, signed_x=True)
    e, d, p = B.expand, B.dw, B.project
    y0, t10, t20 = oracle.block(B.x, (e.weight, e.bias, e.mult, e.shift, -128, 127),
                                (d.weight, d.bias, d.mult, d.shift, -128, 127),
                                (p.weight, p.bias, p.mult, p.shift, p.act_min, p.act_max), 1, True)
    y1, t11, t21 = oracle.block_prelu(B.x, (e.weight, e.bias, e.mult, e.shift, -128, 127, e.mult),
                                      (d.weight, d.bias, d.mult, d.shift, -128, 127, d.mult),
                                      (p.weight, p.bias, p.mult, p.shift, p.act_min, p.act_max), 1, True)
    assert np.array_equal(y0, y1) and np.array_equal(t10, t11) and np.array_equal(t20, t21)
