"""Pins for the CPU oracle: it is checked against things other than itself --
exact rational arithmetic, closed forms, brute force over every ternary matrix on tiny
shapes, library routines on special cases, and values the paper prints."""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from workloads import (make_pw_layer, make_dw_layer, make_block, mobilenetv2_pointwise_layers,
                       mobilenetv2_depthwise_layers, mobilenetv2_param_counts)


# ---------------------------------------------------------------- requantisation
def exact_requant(s, mult, shift):
    """floor(s*mult/2^(31+shift) + 1/2) in exact rationals."""
    v = Fraction(s * mult, 1 << (31 + shift)) + Fraction(1, 2)
    return math.floor(v)


CRAFTED = [(1 << 30, 8), (1 << 30, 0), ((1 << 31) - 1, 14), ((1 << 30) + 1, 9),
           (0x5A5A5A5B, 11), (0x7FFFFFFF, 0), (0x40000000, 31), (0x6DB6DB6E, 13)]


def test_requant_ties_round_toward_plus_infinity():
    # mult = 2^30, shift = 8  =>  scale 2^-9; s = 256 is exactly 0.5
    assert oracle.requant(256, 1 << 30, 8) == 1
    assert oracle.requant(-256, 1 << 30, 8) == 0
    assert oracle.requant(768, 1 << 30, 8) == 2
    assert oracle.requant(-768, 1 << 30, 8) == -1
    assert oracle.requant(255, 1 << 30, 8) == 0
    assert oracle.requant(-257, 1 << 30, 8) == -1
    # mult = 2^30, shift = 0: y = floor(s/2 + 1/2)
    for s in range(-9, 10):
        assert oracle.requant(s, 1 << 30, 0) == math.floor(Fraction(s, 2) + Fraction(1, 2))


@pytest.mark.parametrize("mult,shift", CRAFTED)
def test_requant_exhaustive_small_s(mult, shift):
    for s in range(-(1 << 12), (1 << 12) + 1):
        assert oracle.requant(s, mult, shift) == exact_requant(s, mult, shift)


def test_requant_sampled_wide_s():
    rng = np.random.default_rng(1234)
    for _ in range(20000):
        s = int(rng.integers(-(1 << 21), 1 << 21))
        mult = int(rng.integers(1 << 30, 1 << 31))
        shift = int(rng.integers(0, 32))
        assert oracle.requant(s, mult, shift) == exact_requant(s, mult, shift)
    # extremes of the documented precondition: |s| up to 2^31
    for s in (-(1 << 31), (1 << 31) - 1, -(1 << 31) + 1, 1 << 30, -(1 << 30) - 1):
        for mult, shift in CRAFTED:
            assert oracle.requant(s, mult, shift) == exact_requant(s, mult, shift)


def test_requant_near_every_step_boundary():
    """For a fixed (mult, shift) the output is a step function of s; walk the s values
    around each step (where floor changes) and compare with exact arithmetic."""
    for mult, shift in CRAFTED[:6]:
        den = 1 << (31 + shift)
        for q in range(-130, 131):
            # smallest s with s*mult + den/2 >= q*den
            s0 = -((-(q * den - den // 2)) // mult)  # ceil
            for s in (s0 - 1, s0, s0 + 1):
                if abs(s) < (1 << 31):
                    assert oracle.requant(s, mult, shift) == exact_requant(s, mult, shift)


# ---------------------------------------------------------------- pointwise conv
def py_pw(x, w, bias, mult, shift, lo, hi, res=None):
    """Independent evaluation with Python big ints and Fractions (tiny shapes only)."""
    m, k = x.shape
    nc = w.shape[0]
    out = np.zeros((m, nc), dtype=np.int64)
    for i in range(m):
        for c in range(nc):
            acc = sum(int(x[i, j]) * int(w[c, j]) for j in range(k))
            q = exact_requant(acc + int(bias[c]), int(mult[c]), int(shift[c]))
            q = min(max(q, lo), hi)
            if res is not None:
                q = min(max(q + int(res[i, c]), -128), 127)
            out[i, c] = q
    return out


def test_pw_brute_force_all_ternary_matrices_tiny():
    """K=3, Nc=2: all 3^6 weight matrices, signed inputs incl. -128, against big-int math."""
    x = np.array([[-128, 127, 5], [1, -1, 0], [77, -128, -128], [127, 127, 127]], dtype=np.int8)
    bias = np.array([3, -700], dtype=np.int32)
    mult = np.array([(1 << 30) + 12345, (1 << 31) - 1], dtype=np.int32)
    shift = np.array([0, 2], dtype=np.int32)
    res = np.array([[-64, 63], [100, -100], [0, 1], [-128, 127]], dtype=np.int8)
    for flat in itertools.product((-1, 0, 1), repeat=6):
        w = np.array(flat, dtype=np.int8).reshape(2, 3)
        for r in (None, res):
            got = oracle.pw_conv(x.reshape(1, 2, 2, 3), w, bias, mult, shift, -128, 127,
                                 None if r is None else r.reshape(1, 2, 2, 2))
            want = py_pw(x, w, bias, mult, shift, -128, 127, r)
            assert np.array_equal(got.reshape(4, 2).astype(np.int64), want), (flat, r is None)


def test_pw_zero_weights_give_bias_only():
    L = make_pw_layer(101, 2, 5, 7, 40, 24, signed_x=True)
    w = np.zeros_like(L.weight)
    y = oracle.pw_conv(L.x, w, L.bias, L.mult, L.shift, -128, 127)
    row = np.array([min(max(exact_requant(int(b), int(m), int(s)), -128), 127)
                    for b, m, s in zip(L.bias, L.mult, L.shift)], dtype=np.int8)
    assert np.array_equal(y, np.broadcast_to(row, y.shape))


def test_pw_accum_plus_minus_ones_and_one_hot():
    L = make_pw_layer(102, 1, 6, 6, 33, 33, signed_x=True)
    x2 = L.x.reshape(-1, 33).astype(np.int64)
    ones = np.ones((33, 33), dtype=np.int8)
    acc = oracle.pw_accum(L.x, ones).reshape(-1, 33)
    assert np.array_equal(acc, np.repeat(x2.sum(1, keepdims=True), 33, axis=1))
    acc = oracle.pw_accum(L.x, -ones).reshape(-1, 33)
    assert np.array_equal(acc, -np.repeat(x2.sum(1, keepdims=True), 33, axis=1))
    # one-hot rows select a single input channel; a reversed identity reverses channels
    eye_rev = np.eye(33, dtype=np.int8)[::-1].copy()
    acc = oracle.pw_accum(L.x, eye_rev).reshape(-1, 33)
    assert np.array_equal(acc, x2[:, ::-1])


def test_pw_conv_agrees_with_accum_then_requant():
    """The add/subtract form (sum of selected input channels) equals the product form
    followed by the exact-rational epilogue."""
    L = make_pw_layer(103, 1, 4, 5, 24, 16, signed_x=True, with_residual=True,
                      act_window=(-128, 127))
    acc = oracle.pw_accum(L.x, L.weight).reshape(-1, 16)
    y = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -128, 127, L.residual).reshape(-1, 16)
    r = L.residual.reshape(-1, 16)
    for i in range(acc.shape[0]):
        for c in range(16):
            q = exact_requant(int(acc[i, c]) + int(L.bias[c]), int(L.mult[c]), int(L.shift[c]))
            q = min(max(q, -128), 127)
            q = min(max(q + int(r[i, c]), -128), 127)
            assert y[i, c] == q


def test_pw_accum_matches_library_matmul():
    """Special case that reduces to a library routine: the raw accumulators are an integer
    matrix product."""
    for seed, (k, nc) in enumerate([(24, 144), (64, 384), (960, 160), (17, 5)]):
        L = make_pw_layer(200 + seed, 1, 9, 11, k, nc, signed_x=True)
        acc = oracle.pw_accum(L.x, L.weight).reshape(-1, nc)
        ref = L.x.reshape(-1, k).astype(np.int64) @ L.weight.astype(np.int64).T
        assert np.array_equal(acc.astype(np.int64), ref)


def test_pw_conv_matches_float64_definition_when_exact():
    """Library-routine pin for the whole layer: with float64, s*mult is exact below 2^53,
    so floor(s*mult/2^(31+sh) + 0.5) via numpy int64 arithmetic must agree."""
    L = make_pw_layer(300, 2, 7, 7, 96, 40, with_residual=True, act_window=(-128, 127))
    y = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -128, 127, L.residual)
    acc = L.x.reshape(-1, 96).astype(np.int64) @ L.weight.astype(np.int64).T
    s = acc + L.bias.astype(np.int64)
    num = s * L.mult.astype(np.int64) + (np.int64(1) << (30 + L.shift.astype(np.int64)))
    q = num >> (31 + L.shift.astype(np.int64))  # numpy >> on int64 is an arithmetic (floor) shift
    q = np.clip(q, -128, 127)
    q = np.clip(q + L.residual.reshape(-1, 40).astype(np.int64), -128, 127)
    assert np.array_equal(y.reshape(-1, 40).astype(np.int64), q)


def test_pw_linearity_negation_permutation():
    L = make_pw_layer(104, 1, 5, 5, 48, 20, signed_x=True)
    w = L.weight
    w1 = w.copy(); w1[:, 24:] = 0
    w2 = w.copy(); w2[:, :24] = 0
    a = oracle.pw_accum(L.x, w).astype(np.int64)
    assert np.array_equal(a, oracle.pw_accum(L.x, w1).astype(np.int64) + oracle.pw_accum(L.x, w2))
    assert np.array_equal(-a, oracle.pw_accum(L.x, -w))
    perm = np.random.default_rng(5).permutation(48)
    xp = np.ascontiguousarray(L.x[..., perm])
    wp = np.ascontiguousarray(w[:, perm])
    y0 = oracle.pw_conv(L.x, w, L.bias, L.mult, L.shift, 0, 127)
    y1 = oracle.pw_conv(xp, wp, L.bias, L.mult, L.shift, 0, 127)
    assert np.array_equal(y0, y1)


def test_pw_halving_identity_special_case():
    """mult = 2^30, shift = 0, bias = 0, full window, identity weights: y = floor(x/2 + 1/2)."""
    x = np.arange(-128, 128, dtype=np.int16).astype(np.int8).reshape(1, 16, 16, 1)
    x = np.repeat(x, 8, axis=3)
    w = np.eye(8, dtype=np.int8)
    z = np.zeros(8, dtype=np.int32)
    y = oracle.pw_conv(x, w, z, np.full(8, 1 << 30, np.int32), z, -128, 127)
    want = np.floor(x.astype(np.float64) / 2 + 0.5).astype(np.int8)
    assert np.array_equal(y, want)


def test_pw_clamp_window_and_residual_order():
    """Clamp first, then add the residual with saturation (not the other way round)."""
    x = np.full((1, 1, 1, 4), 127, dtype=np.int8)
    w = np.ones((1, 4), dtype=np.int8)            # acc = 508
    one = np.array([1 << 30], dtype=np.int32)
    zero = np.array([0], dtype=np.int32)
    # scale 1/2 -> q = 254 -> clamp to 100 -> + (-128) = -28
    y = oracle.pw_conv(x, w, zero, one, zero, -5, 100, np.array([-128], np.int8).reshape(1, 1, 1, 1))
    assert int(y.ravel()[0]) == -28
    # saturation of the add
    y = oracle.pw_conv(x, w, zero, one, zero, -5, 100, np.array([127], np.int8).reshape(1, 1, 1, 1))
    assert int(y.ravel()[0]) == 127
    y = oracle.pw_conv(-x, w, zero, one, zero, -128, 100, np.array([-128], np.int8).reshape(1, 1, 1, 1))
    assert int(y.ravel()[0]) == -128


def test_pw_rejects_non_ternary():
    L = make_pw_layer(105, 1, 2, 2, 4, 4)
    w = L.weight.copy(); w[1, 2] = 2
    with pytest.raises(ValueError):
        oracle.pw_conv(L.x, w, L.bias, L.mult, L.shift, 0, 127)


# ---------------------------------------------------------------- depthwise conv
def py_dw(x, w, stride, bias, mult, shift, lo, hi):
    n, h, wd, c = x.shape
    ho = (h - 1) // stride + 1
    wo = (wd - 1) // stride + 1
    out = np.zeros((n, ho, wo, c), dtype=np.int64)
    for b in range(n):
        for oy in range(ho):
            for ox in range(wo):
                for ch in range(c):
                    acc = 0
                    for i in range(3):
                        for j in range(3):
                            iy, ix = oy * stride + i - 1, ox * stride + j - 1
                            if 0 <= iy < h and 0 <= ix < wd:
                                acc += int(x[b, iy, ix, ch]) * int(w[i, j, ch])
                    q = exact_requant(acc + int(bias[ch]), int(mult[ch]), int(shift[ch]))
                    out[b, oy, ox, ch] = min(max(q, lo), hi)
    return out


@pytest.mark.parametrize("h,w,stride", [(3, 3, 1), (4, 5, 1), (4, 5, 2), (5, 4, 2), (1, 1, 1),
                                        (2, 7, 2), (7, 7, 2)])
def test_dw_brute_force_tiny(h, w, stride):
    D = make_dw_layer(400 + h * 10 + w + stride, 2, h, w, 5, stride, signed_x=True,
                      act_window=(-128, 127), shift_range=(2, 6))
    got = oracle.dw_conv(D.x, D.weight, stride, D.bias, D.mult, D.shift, -128, 127)
    want = py_dw(D.x, D.weight, stride, D.bias, D.mult, D.shift, -128, 127)
    assert got.shape == want.shape
    assert np.array_equal(got.astype(np.int64), want)


def test_dw_matches_library_grouped_conv():
    """Special case that reduces to a library routine: accumulators = grouped conv2d
    (float64 is exact here: |acc| <= 9*128*127)."""
    torch = pytest.importorskip("torch")
    for stride in (1, 2):
        D = make_dw_layer(410 + stride, 2, 9, 10, 12, stride, signed_x=True)
        # identity requant with a wide window is impossible in int8, so compare through a
        # scale of exactly 2^-11 (mult=2^30, shift=10) which keeps |q| < 128.
        mult = np.full(12, 1 << 30, np.int32)
        shift = np.full(12, 10, np.int32)
        bias = np.zeros(12, np.int32)
        got = oracle.dw_conv(D.x, D.weight, stride, bias, mult, shift, -128, 127)
        xt = torch.from_numpy(D.x.astype(np.float64)).permute(0, 3, 1, 2)
        wt = torch.from_numpy(D.weight.astype(np.float64)).permute(2, 0, 1).unsqueeze(1)
        acc = torch.nn.functional.conv2d(xt, wt, stride=stride, padding=1, groups=12)
        acc = acc.permute(0, 2, 3, 1).numpy()
        want = np.clip(np.floor(acc / 2048.0 + 0.5), -128, 127).astype(np.int64)
        assert np.array_equal(got.astype(np.int64), want)


def test_dw_closed_forms():
    c = 3
    one = np.full(c, 1 << 30, np.int32)
    zero = np.zeros(c, np.int32)
    # all-ones weights on a constant image: 9v interior, 6v edges, 4v corners; scale 1/2
    x = np.full((1, 5, 6, c), 10, dtype=np.int8)
    w = np.ones((3, 3, c), dtype=np.int8)
    y = oracle.dw_conv(x, w, 1, zero, one, zero, -128, 127)[0, :, :, 0].astype(int)
    assert y[2, 3] == 45 and y[0, 2] == 30 and y[4, 3] == 30 and y[2, 0] == 30
    assert y[0, 0] == 20 and y[4, 5] == 20 and y[0, 5] == 20 and y[4, 0] == 20
    # centre tap only, weight 1: y = floor(x/2 + 1/2) pixel by pixel, any stride
    D = make_dw_layer(420, 1, 6, 7, c, 1, signed_x=True)
    w = np.zeros((3, 3, c), dtype=np.int8); w[1, 1, :] = 1
    y = oracle.dw_conv(D.x, w, 1, zero, one, zero, -128, 127)
    assert np.array_equal(y, np.floor(D.x.astype(np.float64) / 2 + 0.5).astype(np.int8))
    y2 = oracle.dw_conv(D.x, w, 2, zero, one, zero, -128, 127)
    assert np.array_equal(y2, y[:, ::2, ::2, :])
    # a single off-centre tap shifts the image: tap (0,0) reads x[y-1, x-1]
    w = np.zeros((3, 3, c), dtype=np.int8); w[0, 0, :] = 1
    y = oracle.dw_conv(D.x, w, 1, zero, one, zero, -128, 127)
    half = np.floor(D.x.astype(np.float64) / 2 + 0.5).astype(np.int8)
    assert np.array_equal(y[:, 1:, 1:, :], half[:, :-1, :-1, :])
    assert not y[:, 0, :, :].any() and not y[:, :, 0, :].any()


# ---------------------------------------------------------------- block
def test_block_is_the_three_layers_chained():
    B = make_block(500, 2, 6, 6, 8, 6)
    e, d, p = B.expand, B.dw, B.project
    y, t1, t2 = oracle.block(B.x, (e.weight, e.bias, e.mult, e.shift, 0, 127),
                             (d.weight, d.bias, d.mult, d.shift, 0, 127),
                             (p.weight, p.bias, p.mult, p.shift, -128, 127), 1, True)
    a = oracle.pw_conv(B.x, e.weight, e.bias, e.mult, e.shift, 0, 127)
    b = oracle.dw_conv(a, d.weight, 1, d.bias, d.mult, d.shift, 0, 127)
    c = oracle.pw_conv(b, p.weight, p.bias, p.mult, p.shift, -128, 127, B.x)
    assert np.array_equal(t1, a) and np.array_equal(t2, b) and np.array_equal(y, c)
    # and against the big-int evaluation end to end on this tiny block
    a2 = py_pw(B.x.reshape(-1, 8), e.weight, e.bias, e.mult, e.shift, 0, 127)
    b2 = py_dw(a2.reshape(2, 6, 6, 48), d.weight, 1, d.bias, d.mult, d.shift, 0, 127)
    c2 = py_pw(b2.reshape(-1, 48), p.weight, p.bias, p.mult, p.shift, -128, 127, B.x.reshape(-1, 8))
    assert np.array_equal(y.reshape(-1, 8).astype(np.int64), c2)


# ---------------------------------------------------------------- structure pins from the paper
def test_layer_enumeration_matches_paper_parameter_shares(paper_values):
    pw = mobilenetv2_pointwise_layers()
    dw = mobilenetv2_depthwise_layers()
    assert len(pw) == 34 and len(dw) == 17
    counts = mobilenetv2_param_counts()
    total = counts["pointwise"] + counts["depthwise"] + counts["stem"] + counts["classifier"]
    assert counts["pointwise"] == 2124672
    pw_share = 100.0 * counts["pointwise"] / total
    dw_share = 100.0 * counts["depthwise"] / total
    assert round(pw_share, 1) == paper_values["pointwise_param_share_pct"]
    assert round(dw_share, 1) == paper_values["depthwise_param_share_pct"]
    assert sum(p.residual for p in pw) == 10


def test_two_bit_storage_matches_paper_model_sizes(paper_values):
    """2 bits per ternary weight + int8 elsewhere + fp16 BatchNorm reproduces the paper's
    1.95 MB; everything in fp16 reproduces its 7.01 MB."""
    c = mobilenetv2_param_counts()
    others = c["depthwise"] + c["stem"] + c["classifier"]
    prom_mb = (c["pointwise"] * 2 / 8 + others * 1 + c["batchnorm_affine"] * 2) / 1e6
    fp16_mb = (c["pointwise"] + others + c["batchnorm_affine"]) * 2 / 1e6
    assert abs(prom_mb - paper_values["prom_model_size_mb"]) < 0.02
    assert abs(fp16_mb - paper_values["fp16_model_size_mb"]) < 0.01
    # 1.58 bits per weight would not reproduce it
    alt_mb = (c["pointwise"] * 1.58 / 8 + others + c["batchnorm_affine"] * 2) / 1e6
    assert abs(alt_mb - paper_values["prom_model_size_mb"]) > 0.05


def test_generator_distributions(paper_values):
    L = make_pw_layer(600, 4, 14, 14, 64, 384)
    assert L.x.min() == 0 and L.x.max() == 127
    frac = np.bincount(L.weight.ravel().astype(np.int64) + 1) / L.weight.size
    assert abs(frac[1] - 0.5) < 0.01 and abs(frac[0] - 0.25) < 0.01 and abs(frac[2] - 0.25) < 0.01
    assert L.bias.min() >= -(1 << 12) and L.bias.max() <= (1 << 12)
    assert L.mult.min() >= (1 << 30) and L.shift.min() >= 8 and L.shift.max() <= 14
    # the init-time distribution of the paper as an alternative zero fraction
    L2 = make_pw_layer(601, 1, 2, 2, 256, 512, p_zero=paper_values["init_zero_fraction"])
    frac = np.bincount(L2.weight.ravel().astype(np.int64) + 1) / L2.weight.size
    assert abs(frac[1] - paper_values["init_zero_fraction"]) < 0.01
    assert abs(frac[0] - paper_values["init_plus_fraction"]) < 0.01
    assert abs(frac[2] - paper_values["init_plus_fraction"]) < 0.01
    # same seed -> same tensors; different seed -> different
    L3 = make_pw_layer(600, 4, 14, 14, 64, 384)
    assert np.array_equal(L.x, L3.x) and np.array_equal(L.weight, L3.weight)
    assert not np.array_equal(L.x, make_pw_layer(602, 4, 14, 14, 64, 384).x)
