"""Parity of the PReLU requantisation (mult_neg in the requantisation parameters) in every
kernel that has an epilogue, against the CPU oracle: bit-exact."""
import numpy as np
import pytest

import oracle
from workloads import make_pw_layer, make_dw_layer, make_block, prelu_mult_neg
from gpu_util import assert_same, dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def _rq(P, L, mneg, window=(-128, 127)):
    return P.Requant(dev(L.bias), dev(L.mult), dev(L.shift), window[0], window[1], dev(mneg))


def _run_pw(P, L, mneg, plan=None, window=(-128, 127), residual=True):
    torch = torch_cuda()
    res = dev(L.residual) if (residual and L.residual is not None) else None
    args = (dev(L.x), dev(P.prom_pack_ternary(L.weight)), L.cout, _rq(P, L, mneg, window), res)
    y = P.prom_pw_conv(*args) if plan is None else P.prom_pw_conv_ex(*args, plan=plan)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def _want_pw(L, mneg, window=(-128, 127), residual=True):
    return oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, window[0], window[1],
                          residual=L.residual if residual else None, mult_neg=mneg)


PW_SHAPES = [
    # n, h, w, cin, cout: one chunk, several chunks, whole rows from one workgroup, ragged widths,
    # one pixel, 8-byte loads (cin % 16 == 8), the generic kernel (odd channel counts)
    (2, 28, 28, 16, 96), (2, 14, 14, 96, 576), (3, 9, 13, 32, 192), (2, 7, 7, 160, 960), (1, 1, 1, 64, 64),
    (2, 11, 5, 24, 144), (1, 6, 7, 72, 40), (2, 5, 5, 320, 1280), (1, 17, 3, 48, 20), (2, 4, 9, 5, 7),
    (1, 3, 3, 33, 130), (64, 14, 14, 64, 384), (32, 28, 28, 32, 192),
]


@pytest.mark.parametrize("shape", PW_SHAPES)
@pytest.mark.parametrize("res", [False, True])
def test_pw_prelu_shapes(P, shape, res):
    n, h, w, cin, cout = shape
    L = make_pw_layer(11000 + cin + cout, n, h, w, cin, cout, signed_x=True, with_residual=res,
                      shift_range=(3, 8))
    mneg = prelu_mult_neg(11000 + cin, L.mult)
    assert_same(_run_pw(P, L, mneg), _want_pw(L, mneg), f"pw prelu {shape} res={res}")


def test_pw_prelu_every_shift_extreme_multipliers_and_window(P):
    """Shifts 0..31, multipliers at the ends of the int32 range, a narrow window."""
    L = make_pw_layer(11100, 2, 9, 9, 64, 128, signed_x=True, shift_range=(0, 31))
    mneg = prelu_mult_neg(11100, L.mult)
    mneg[::5] = -(1 << 31)
    mneg[1::5] = (1 << 31) - 1
    mneg[2::5] = 0
    L.bias[::3] *= 4000
    for window in ((-128, 127), (-7, 19), (0, 127)):
        assert_same(_run_pw(P, L, mneg, window=window), _want_pw(L, mneg, window), f"window {window}")


def test_pw_prelu_equal_multipliers_reproduce_the_plain_layer(P):
    torch = torch_cuda()
    L = make_pw_layer(11200, 2, 12, 12, 32, 192, signed_x=True, with_residual=True)
    plain = P.prom_pw_conv(dev(L.x), dev(P.prom_pack_ternary(L.weight)), L.cout,
                           P.Requant(dev(L.bias), dev(L.mult), dev(L.shift), -128, 127), dev(L.residual))
    torch.cuda.synchronize()
    assert_same(_run_pw(P, L, L.mult.copy()), plain.cpu().numpy(), "slope 1")


@pytest.mark.parametrize("nt", list(range(1, 11)))
def test_pw_prelu_every_tile_plan(P, nt):
    for pt in (1, 2, 4):
        if (pt == 2 and nt > 6) or (pt == 4 and nt > 2):
            continue
        for (cin, cout) in ((32, 16 * nt), (80, 16 * nt * 2 + 16), (24, 16 * nt)):
            L = make_pw_layer(11300 + nt * 7 + pt, 2, 9, 11, cin, cout, signed_x=True,
                              with_residual=(cin == 80), shift_range=(0, 9))
            mneg = prelu_mult_neg(11300 + nt, L.mult)
            assert_same(_run_pw(P, L, mneg, plan=P.PwPlan(nt, pt, 0, 0)), _want_pw(L, mneg),
                        f"nt={nt} pt={pt} {cin}->{cout}")


@pytest.mark.parametrize("cw", [2, 3, 4])
def test_pw_prelu_row_cooperative_plans(P, cw):
    for nt in range(1, 7):
        cout = 16 * nt * cw
        for (n, h, w, cin) in ((2, 9, 13, 32), (1, 7, 7, 160), (2, 6, 9, 24)):
            L = make_pw_layer(11400 + 10 * nt + cw + cin, n, h, w, cin, cout, signed_x=True,
                              with_residual=(cin == 32), shift_range=(0, 9))
            mneg = prelu_mult_neg(11400 + nt + cw, L.mult)
            assert_same(_run_pw(P, L, mneg, plan=P.PwPlan(nt, 0, 0, cw)), _want_pw(L, mneg),
                        f"rows cw={cw} nt={nt} cin={cin}")


def test_addsub_design_refuses_prelu(P):
    L = make_pw_layer(11500, 1, 4, 4, 32, 16)
    with pytest.raises(P.PromError) as e:
        P.prom_pw_conv_addsub(dev(L.x), dev(P.prom_pack_ternary(L.weight)), L.cout, _rq(P, L, L.mult.copy()), None)
    assert e.value.code == -2


def test_sequence_mixes_prelu_and_plain_layers(P):
    """Shared launches that hold PReLU and plain layers side by side (the expand layers of a PReLU
    network have the activation, the project layers have none), small and large layers."""
    torch = torch_cuda()
    n = 64
    shapes = [(112, 32, 16, False), (112, 16, 96, True), (56, 24, 144, True), (56, 96, 24, False),
              (14, 64, 384, True), (7, 160, 960, True), (14, 384, 64, False), (7, 960, 160, False),
              (28, 32, 192, True), (7, 320, 1280, True)]
    classes = [P.prom_pw_batch_class(n, hw, hw, cin, cout) for hw, cin, cout, _ in shapes]
    assert 1 in classes and 2 in classes
    layers, wants = [], []
    for i, (hw, cin, cout, prelu) in enumerate(shapes):
        L = make_pw_layer(11600 + i, n, hw, hw, cin, cout, signed_x=True, act_window=(-128, 127),
                          shift_range=(2, 7))
        mneg = prelu_mult_neg(11600 + i, L.mult) if prelu else None
        rq = _rq(P, L, mneg) if prelu else P.Requant(dev(L.bias), dev(L.mult), dev(L.shift), -128, 127)
        y = torch.full((n, hw, hw, cout), -99, dtype=torch.int8, device="cuda")
        layers.append((dev(L.x), dev(P.prom_pack_ternary(L.weight)), cout, rq, None, y))
        wants.append(dev(oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -128, 127, mult_neg=mneg)))
    seq = P.PwSequence(layers)
    for run in range(2):
        for l in layers:
            l[5].fill_(-99)
        seq.run()
        torch.cuda.synchronize()
        for (hw, cin, cout, prelu), l, want in zip(shapes, layers, wants):
            assert int((l[5] != want).sum()) == 0, f"run {run}: {cin}->{cout} @ {hw} prelu={prelu}"


def test_sequence_expansion_layers_with_prelu(P):
    """The body of the shared launch that keeps a pixel group's activations in registers and walks
    over the output channels, for PReLU layers: one to three k steps, one to five parts, ragged
    pixel units, shift 0, most negative and zero negative-side multipliers, next to plain members
    that take the same body and members that take the streaming bodies."""
    torch = torch_cuda()
    cases = [  # n, h, w, cin, cout, shift_range, prelu
        (3, 7, 9, 32, 192, (3, 8), True), (2, 14, 14, 64, 384, (0, 8), True), (5, 5, 5, 16, 64 * 9, (2, 6), False),
        (1, 31, 3, 48, 64 * 10, (0, 4), True), (3, 14, 14, 96, 576, (3, 8), True), (2, 9, 11, 128, 64 * 11, (1, 7), True),
        (4, 7, 7, 160, 960, (3, 8), True), (1, 13, 13, 192, 64 * 7, (0, 3), True), (2, 6, 7, 144, 128, (2, 9), False),
        (1, 1, 1, 64, 128, (3, 8), True), (2, 7, 7, 320, 1280, (3, 8), True), (3, 7, 9, 64, 96, (3, 8), True),
        (3, 7, 9, 384, 64, (3, 8), False),
    ]
    layers, wants = [], []
    for i, (n, h, w, cin, cout, sr, prelu) in enumerate(cases):
        L = make_pw_layer(11900 + i, n, h, w, cin, cout, signed_x=True, act_window=(-128, 127), shift_range=sr)
        mneg = None
        if prelu:
            mneg = prelu_mult_neg(11900 + i, L.mult)
            mneg[::7] = -(1 << 31)
            mneg[3::11] = 0
        rq = _rq(P, L, mneg) if prelu else P.Requant(dev(L.bias), dev(L.mult), dev(L.shift), -128, 127)
        y = torch.full((n, h, w, cout), -99, dtype=torch.int8, device="cuda")
        layers.append((dev(L.x), dev(P.prom_pack_ternary(L.weight)), cout, rq, None, y))
        wants.append(oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -128, 127, mult_neg=mneg))
    seq = P.PwSequence(layers)
    for run in range(2):
        for l in layers:
            l[5].fill_(-99)
        seq.run()
        torch.cuda.synchronize()
        for c, l, want in zip(cases, layers, wants):
            assert_same(l[5].cpu().numpy(), want, f"run {run}: case {c}")


def test_sequence_large_wide_row_layers_with_prelu(P):
    """24 -> 144 at high resolution with PReLU inside the launch of large layers (the body where one
    wavefront assembles whole rows): shift ranges from 0 and from 2, ragged pixel counts, most
    negative, largest and zero negative-side multipliers, a plain neighbour."""
    torch = torch_cuda()
    cases = [(65, 56, 55, 24, 144, (2, 9), True), (37, 113, 57, 24, 144, (0, 5), True),
             (64, 56, 56, 24, 144, (2, 3), True), (64, 112, 112, 16, 96, (2, 7), False)]
    assert [P.prom_pw_batch_class(n, h, w, ci, co) for n, h, w, ci, co, _, _ in cases] == [2, 2, 2, 2]
    layers, wants = [], []
    for i, (n, h, w, cin, cout, sr, prelu) in enumerate(cases):
        L = make_pw_layer(12300 + i, n, h, w, cin, cout, signed_x=True, act_window=(-128, 127), shift_range=sr)
        mneg = None
        if prelu:
            mneg = prelu_mult_neg(12300 + i, L.mult)
            mneg[::7] = -(1 << 31)
            mneg[3::11] = 0
            mneg[5::13] = (1 << 31) - 1
        rq = _rq(P, L, mneg) if prelu else P.Requant(dev(L.bias), dev(L.mult), dev(L.shift), -128, 127)
        y = torch.full((n, h, w, cout), -99, dtype=torch.int8, device="cuda")
        layers.append((dev(L.x), dev(P.prom_pack_ternary(L.weight)), cout, rq, None, y))
        wants.append(dev(oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -128, 127, mult_neg=mneg)))
    seq = P.PwSequence(layers)
    for run in range(2):
        for l in layers:
            l[5].fill_(-99)
        seq.run()
        torch.cuda.synchronize()
        for c, l, want in zip(cases, layers, wants):
            assert int((l[5] != want).sum()) == 0, f"run {run}: case {c}"


DW_SHAPES = [(2, 4, 5, 12, 1), (2, 4, 5, 12, 2), (1, 7, 7, 960, 1), (3, 14, 14, 384, 1), (2, 28, 28, 192, 2),
             (1, 9, 11, 20, 2), (2, 5, 4, 5, 1), (2, 5, 4, 7, 2), (1, 13, 10, 4, 2), (8, 56, 56, 144, 1)]


@pytest.mark.parametrize("shape", DW_SHAPES)
def test_dw_prelu_shapes(P, shape):
    torch = torch_cuda()
    n, h, w, c, stride = shape
    D = make_dw_layer(12000 + h * 31 + c + stride, n, h, w, c, stride, signed_x=True,
                      act_window=(-128, 127), shift_range=(0, 12))
    mneg = prelu_mult_neg(12000 + c, D.mult)
    mneg[::7] = -(1 << 31)
    want = oracle.dw_conv(D.x, D.weight, stride, D.bias, D.mult, D.shift, -128, 127, mult_neg=mneg)
    y = P.prom_dw_conv(dev(D.x), dev(D.weight), stride, _rq(P, D, mneg))
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), want, f"dw prelu {shape}")
    if c % 4 == 0:
        # a negative-side array that is not 16-byte aligned: the one-thread-per-output kernel
        off = dev(np.concatenate([np.zeros(1, np.int32), mneg]))[1:]
        rq = P.Requant(dev(D.bias), dev(D.mult), dev(D.shift), -128, 127, off)
        y = P.prom_dw_conv(dev(D.x), dev(D.weight), stride, rq)
        torch.cuda.synchronize()
        assert_same(y.cpu().numpy(), want, f"dw prelu unaligned {shape}")


def _block_prelu(P, B, seed, path=0):
    torch = torch_cuda()
    e, d, p = B.expand, B.dw, B.project
    ne, nd = prelu_mult_neg(seed, e.mult), prelu_mult_neg(seed + 1, d.mult)
    ws = torch.empty(P.prom_block_workspace_size(B.n, B.h, B.w, B.cin, B.chid, B.cout, B.stride),
                     dtype=torch.int8, device="cuda")
    y = P.prom_block(dev(B.x), B.chid, B.cout, B.stride,
                     dev(P.prom_pack_ternary(e.weight)), _rq(P, e, ne),
                     dev(d.weight), _rq(P, d, nd),
                     dev(P.prom_pack_ternary(p.weight)),
                     P.Requant(dev(p.bias), dev(p.mult), dev(p.shift), p.act_min, p.act_max),
                     B.add_residual, ws, path=path)
    torch.cuda.synchronize()
    want, _, _ = oracle.block_prelu(B.x, (e.weight, e.bias, e.mult, e.shift, -128, 127, ne),
                                    (d.weight, d.bias, d.mult, d.shift, -128, 127, nd),
                                    (p.weight, p.bias, p.mult, p.shift, p.act_min, p.act_max),
                                    B.stride, B.add_residual)
    return y.cpu().numpy(), want


@pytest.mark.parametrize("shape", [
    # n, h, w, cin, t, cout, stride; the first rows run the fused kernel, the last the three launches
    (2, 9, 9, 16, 6, 16, 1), (1, 14, 14, 24, 6, 32, 2), (2, 7, 7, 160, 6, 320, 1), (3, 13, 17, 16, 9, 16, 1),
    (1, 28, 28, 32, 6, 64, 1), (2, 15, 13, 16, 5, 24, 2), (1, 5, 6, 8, 1, 8, 1), (16, 56, 56, 24, 6, 24, 1),
    (2, 14, 14, 64, 6, 64, 1), (80, 56, 56, 24, 6, 24, 1), (2, 7, 7, 160, 6, 160, 1), (1, 7, 7, 320, 6, 320, 1),
])
def test_block_prelu_shapes(P, shape):
    n, h, w, cin, t, cout, stride = shape
    B = make_block(13000 + cin + cout, n, h, w, cin, t, cout, stride, signed_x=True,
                   expand_shift=(3, 6), dw_shift=(8, 10), project_shift=(3, 6))
    paths = [P.BLOCK_UNFUSED, P.BLOCK_AUTO]
    if P.prom_block_can_fuse(n, h, w, cin, cin * t, cout, stride):
        paths.append(P.BLOCK_FUSED)
    for path in paths:
        got, want = _block_prelu(P, B, 13000 + cin, path)
        assert_same(got, want, f"block prelu {shape} path={path}")


def test_block_prelu_covers_both_paths(P):
    assert P.prom_block_can_fuse(2, 9, 9, 16, 96, 16, 1) and P.prom_block_can_fuse(16, 56, 56, 24, 144, 24, 1)
    assert not P.prom_block_can_fuse(2, 14, 14, 64, 384, 64, 1)
