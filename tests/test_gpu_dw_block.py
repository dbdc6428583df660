"""Parity of prom_dw_conv and prom_block against the CPU oracle: bit-exact."""
import numpy as np
import pytest

import oracle
from workloads import make_dw_layer, make_pw_layer, make_block, BASELINE_CONFIGS, CONFIG_SEED_BASE
from gpu_util import assert_same, dev, requant_dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


DW_SHAPES = [
    # n, h, w, c, stride
    (1, 1, 1, 4, 1), (1, 3, 3, 8, 1), (2, 4, 5, 12, 1), (2, 4, 5, 12, 2), (1, 7, 7, 960, 1),
    (3, 14, 14, 384, 1), (2, 28, 28, 192, 2), (1, 9, 11, 20, 2), (1, 112, 112, 32, 1),
    (1, 56, 56, 144, 2), (2, 5, 4, 5, 1), (2, 5, 4, 7, 2), (1, 2, 7, 1, 2), (1, 15, 1, 16, 2),
    # row groups of 4 with 1, 2, 3 rows left over, both strides, even and odd sizes
    (2, 5, 6, 8, 1), (2, 6, 6, 8, 2), (1, 7, 3, 24, 1), (1, 13, 10, 4, 2), (3, 10, 9, 36, 1),
    (1, 12, 12, 64, 2), (2, 1, 9, 8, 1), (2, 9, 1, 8, 1), (2, 2, 2, 4, 2),
]


@pytest.mark.parametrize("shape", DW_SHAPES)
def test_dw_shapes(P, shape):
    torch = torch_cuda()
    n, h, w, c, stride = shape
    D = make_dw_layer(5000 + h * 31 + c + stride, n, h, w, c, stride, signed_x=True,
                      act_window=(-128, 127), shift_range=(4, 10))
    D.x.reshape(-1)[::29] = -128
    y = P.prom_dw_conv(dev(D.x), dev(D.weight), stride, requant_dev(P, D))
    torch.cuda.synchronize()
    want = oracle.dw_conv(D.x, D.weight, stride, D.bias, D.mult, D.shift, -128, 127)
    assert_same(y.cpu().numpy(), want, f"dw {shape}")


def test_dw_full_shift_range_and_unaligned_parameters(P):
    """Shifts from 0 to 31 (the kernel takes the general form of the requantisation), and
    parameter arrays that are not 16-byte aligned (the one-thread-per-output kernel takes over)."""
    torch = torch_cuda()
    D = make_dw_layer(5050, 2, 11, 13, 40, 1, signed_x=True, act_window=(-128, 127), shift_range=(0, 31))
    want = oracle.dw_conv(D.x, D.weight, 1, D.bias, D.mult, D.shift, -128, 127)
    y = P.prom_dw_conv(dev(D.x), dev(D.weight), 1, requant_dev(P, D))
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), want, "dw shifts 0..31")
    for seed, shape, stride, sr in ((5051, (2, 11, 13, 40), 2, (0, 31)), (5052, (3, 17, 9, 64), 1, (0, 2)),
                                    (5053, (3, 17, 9, 64), 2, (0, 1)), (5054, (2, 5, 9, 24), 1, (0, 3))):
        D2 = make_dw_layer(seed, *shape, stride, signed_x=True, act_window=(-128, 127), shift_range=sr)
        y2 = P.prom_dw_conv(dev(D2.x), dev(D2.weight), stride, requant_dev(P, D2))
        torch.cuda.synchronize()
        assert_same(y2.cpu().numpy(), oracle.dw_conv(D2.x, D2.weight, stride, D2.bias, D2.mult, D2.shift, -128, 127),
                    f"dw {shape} stride {stride} shifts {sr}")
    pad = lambda a: dev(np.concatenate([np.zeros(1, a.dtype), a]))[1:]
    rq = P.Requant(pad(D.bias), pad(D.mult), pad(D.shift), -128, 127)
    y = P.prom_dw_conv(dev(D.x), dev(D.weight), 1, rq)
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), want, "dw unaligned parameters")


def test_dw_full_size_layer_every_output(P):
    """A full-size layer of the batch-128 sweep (56x56x144, both strides), every output."""
    torch = torch_cuda()
    for stride in (1, 2):
        D = make_dw_layer(5060 + stride, 128, 56, 56, 144, stride)
        want = dev(oracle.dw_conv(D.x, D.weight, stride, D.bias, D.mult, D.shift, D.act_min, D.act_max))
        x, w, rq = dev(D.x), dev(D.weight), requant_dev(P, D)
        for run in range(3):
            y = P.prom_dw_conv(x, w, stride, rq)
            torch.cuda.synchronize()
            bad = int((y != want).sum())
            assert bad == 0, f"stride {stride}, run {run}: {bad} outputs differ"


def test_dw_relu6_window(P):
    torch = torch_cuda()
    D = make_dw_layer(5100, 4, 28, 28, 192, 1)
    y = P.prom_dw_conv(dev(D.x), dev(D.weight), 1, requant_dev(P, D))
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), oracle.dw_conv(D.x, D.weight, 1, D.bias, D.mult, D.shift, 0, 127), "dw relu6")


def _run_block(P, B, path=0):
    torch = torch_cuda()
    e, d, p = B.expand, B.dw, B.project
    ws = torch.empty(P.prom_block_workspace_size(B.n, B.h, B.w, B.cin, B.chid, B.cout, B.stride),
                     dtype=torch.int8, device="cuda")
    y = P.prom_block(dev(B.x), B.chid, B.cout, B.stride,
                     dev(P.prom_pack_ternary(e.weight)), requant_dev(P, e),
                     dev(d.weight), requant_dev(P, d),
                     dev(P.prom_pack_ternary(p.weight)), requant_dev(P, p),
                     B.add_residual, ws, path=path)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def _oracle_block(B):
    e, d, p = B.expand, B.dw, B.project
    y, _, _ = oracle.block(B.x, (e.weight, e.bias, e.mult, e.shift, e.act_min, e.act_max),
                           (d.weight, d.bias, d.mult, d.shift, d.act_min, d.act_max),
                           (p.weight, p.bias, p.mult, p.shift, p.act_min, p.act_max),
                           B.stride, B.add_residual)
    return y


def test_block_config4_full_output(P):
    c = BASELINE_CONFIGS[4]
    B = make_block(CONFIG_SEED_BASE + 4, c["n"], c["h"], c["w"], c["cin"], c["t"], stride=c["stride"])
    assert B.add_residual
    assert P.prom_block_is_fused(c["n"], c["h"], c["w"], c["cin"], c["cin"] * c["t"], c["cin"], c["stride"])
    want = _oracle_block(B)
    assert_same(_run_block(P, B), want, "config 4")
    assert_same(_run_block(P, B, P.BLOCK_UNFUSED), want, "config 4, three launches")


@pytest.mark.parametrize("shape", [
    # n, h, w, cin, t, cout, stride
    (2, 9, 9, 16, 6, 16, 1), (1, 14, 14, 24, 6, 32, 2), (2, 7, 7, 160, 6, 320, 1), (1, 5, 6, 8, 1, 8, 1),
    (1, 112, 112, 16, 6, 24, 2),
    # fused-kernel corner cases: ragged last band, hidden width off the 64-channel chunk (144, 80),
    # 17-wide rows, stride 2 on odd sizes, cout below and above one tile, no skip, one pixel
    (3, 13, 17, 16, 9, 16, 1), (2, 15, 13, 16, 5, 24, 2), (1, 28, 28, 32, 6, 64, 1), (2, 1, 1, 16, 4, 16, 1),
    (1, 33, 9, 48, 3, 48, 1), (1, 56, 56, 32, 6, 32, 2), (2, 6, 40, 64, 2, 40, 1), (1, 3, 300, 16, 2, 16, 1),
    # 24 and 40 input channels (pixels padded to 16 bytes in LDS), wide outputs (6 and 10 projection
    # tiles), 3 chunks with a ragged last one, the smallest and a single-row image
    (2, 28, 28, 24, 6, 24, 1), (1, 17, 9, 40, 4, 96, 2), (2, 7, 7, 32, 6, 160, 1), (1, 14, 14, 24, 7, 136, 1),
    (3, 1, 1, 16, 6, 16, 1), (1, 1, 37, 32, 5, 32, 1), (1, 37, 1, 32, 5, 32, 2),
    # more than 3 chunks of hidden channels (4, 5, 6, 9, 15 chunks, ragged last chunk, every
    # projection width class, both strides): the fully fused kernel refuses these, the two-launch
    # form (depthwise and projection fused) takes them
    (2, 14, 14, 64, 6, 64, 1), (2, 14, 14, 64, 6, 96, 1), (2, 14, 14, 96, 6, 96, 1), (1, 14, 14, 96, 6, 160, 2),
    (2, 7, 7, 160, 6, 160, 1), (1, 9, 11, 64, 5, 32, 1), (1, 10, 6, 40, 7, 24, 2), (3, 5, 5, 128, 2, 128, 1),
])
def test_block_shapes(P, shape):
    n, h, w, cin, t, cout, stride = shape
    B = make_block(6000 + cin + cout, n, h, w, cin, t, cout, stride, signed_x=True)
    want = _oracle_block(B)
    # both forms of the block whatever the library would pick for the shape, then its own choice
    if P.prom_block_can_fuse(n, h, w, cin, cin * t, cout, stride):
        assert_same(_run_block(P, B, P.BLOCK_FUSED), want, f"block {shape} fused")
    else:
        with pytest.raises(P.PromError) as e:
            _run_block(P, B, P.BLOCK_FUSED)
        assert e.value.code == -2
    assert_same(_run_block(P, B, P.BLOCK_UNFUSED), want, f"block {shape} three launches")
    # expand, then depthwise and projection in one kernel
    if P.prom_dw_pw_can_fuse(n, h, w, cin * t, cout, stride):
        assert_same(_run_block(P, B, P.BLOCK_DWPROJ), want, f"block {shape} two launches")
    else:
        with pytest.raises(P.PromError) as e:
            _run_block(P, B, P.BLOCK_DWPROJ)
        assert e.value.code == -2
    # one kernel with the expanded band resident in LDS as 16-channel planes
    if P.prom_block_planes_applies(n, h, w, cin, cin * t, cout, stride):
        assert_same(_run_block(P, B, P.BLOCK_PLANES), want, f"block {shape} plane-resident kernel")
    else:
        with pytest.raises(P.PromError) as e:
            _run_block(P, B, P.BLOCK_PLANES)
        assert e.value.code == -2
    assert_same(_run_block(P, B), want, f"block {shape}")


def test_block_forms_and_queries(P):
    """What prom_block picks: one kernel for deep blocks on small maps and for small problems, three
    launches for large maps at a large batch; the limits of the two one-kernel forms."""
    assert P.prom_block_is_fused(64, 28, 28, 32, 192, 32, 1) and P.prom_block_is_fused(128, 28, 28, 32, 192, 64, 2)
    assert P.prom_block_is_fused(128, 14, 14, 64, 384, 64, 1) and P.prom_block_is_fused(128, 7, 7, 160, 960, 320, 1)
    assert P.prom_block_is_fused(2, 9, 9, 16, 96, 16, 1) and P.prom_block_can_fuse(2, 9, 9, 16, 96, 16, 1)
    assert not P.prom_block_is_fused(128, 112, 112, 16, 96, 24, 2) and P.prom_block_can_fuse(128, 112, 112, 16, 96, 24, 2)
    assert P.prom_block_planes_applies(128, 112, 112, 16, 96, 24, 2)
    assert not P.prom_block_can_fuse(2, 14, 14, 64, 384, 64, 1)      # 6 chunks of hidden channels
    assert P.prom_block_planes_applies(2, 14, 14, 64, 384, 64, 1)
    assert not P.prom_block_can_fuse(2, 7, 7, 32, 192, 320, 1)       # 320 output channels
    assert P.prom_block_planes_applies(2, 7, 7, 32, 192, 320, 1)
    assert not P.prom_block_can_fuse(2, 7, 7, 12, 72, 16, 1)         # cin % 8 != 0
    assert not P.prom_block_planes_applies(2, 7, 7, 12, 72, 16, 1)
    assert not P.prom_block_planes_applies(1, 14, 14, 24, 168, 136, 1)  # hidden channels not a multiple of 16
    assert not P.prom_block_planes_applies(1, 14, 14, 200, 1600, 200, 1)  # more than 192 input channels
    assert P.prom_block_can_fuse(1, 28, 28, 24, 144, 24, 1)          # 24 input channels: padded pixels


DWPW_SHAPES = [
    # n, h, w, c, cout, stride, residual
    (2, 14, 14, 384, 64, 1, True), (3, 14, 14, 576, 96, 1, True), (2, 14, 14, 576, 160, 2, False),
    (3, 7, 7, 960, 160, 1, True), (2, 7, 7, 960, 320, 1, False), (40, 14, 14, 384, 96, 1, False),
    (80, 7, 7, 960, 160, 1, True), (1, 1, 1, 64, 16, 1, True), (1, 1, 9, 16, 8, 1, False), (2, 9, 1, 32, 4, 2, False),
    # ragged last chunk of hidden channels (144, 80, 208), bands with a ragged last one, wide rows,
    # stride 2 on odd and even sizes, every projection width class
    (2, 12, 12, 144, 24, 1, True), (1, 13, 17, 80, 40, 2, False), (2, 28, 28, 192, 32, 1, True),
    (1, 28, 28, 192, 64, 2, False), (1, 56, 56, 144, 24, 1, True), (1, 5, 85, 48, 16, 1, False),
    (2, 15, 11, 208, 112, 2, False), (1, 7, 7, 128, 320, 1, True), (5, 6, 7, 320, 200, 1, False),
    (1, 30, 85, 32, 16, 1, False),
]


@pytest.mark.parametrize("shape", DWPW_SHAPES)
def test_dw_pw_fused_shapes(P, shape):
    """prom_dw_pw_conv (depthwise 3x3 and the projection behind it in one kernel) against the
    oracle's depthwise layer followed by its pointwise layer, every output."""
    torch = torch_cuda()
    n, h, w, c, cout, stride, res = shape
    ho, wo = (h - 1) // stride + 1, (w - 1) // stride + 1
    D = make_dw_layer(7100 + c + cout, n, h, w, c, stride, signed_x=True, act_window=(0, 127), shift_range=(4, 10))
    Q = make_pw_layer(7200 + c + cout, n, ho, wo, c, cout, act_window=(-128, 127), shift_range=(5, 9),
                      with_residual=res, make_x=False)
    assert P.prom_dw_pw_can_fuse(n, h, w, c, cout, stride)
    mid = oracle.dw_conv(D.x, D.weight, stride, D.bias, D.mult, D.shift, 0, 127)
    want = oracle.pw_conv(mid, Q.weight, Q.bias, Q.mult, Q.shift, -128, 127, Q.residual if res else None)
    y = torch.full((n, ho, wo, cout), -99, dtype=torch.int8, device="cuda")
    P.prom_dw_pw_conv(dev(D.x), dev(D.weight), stride, requant_dev(P, D), dev(P.prom_pack_ternary(Q.weight)), cout,
                      requant_dev(P, Q), dev(Q.residual) if res else None, y)
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), want, f"dw+pw {shape}")
    if res:  # the residual read from the output buffer itself
        yb = dev(Q.residual)
        P.prom_dw_pw_conv(dev(D.x), dev(D.weight), stride, requant_dev(P, D), dev(P.prom_pack_ternary(Q.weight)),
                          cout, requant_dev(P, Q), yb, yb)
        torch.cuda.synchronize()
        assert_same(yb.cpu().numpy(), want, f"dw+pw {shape}, residual in place")


def test_dw_pw_fused_shift_zero_prelu_and_limits(P):
    """Shifts from 0 up in both layers, PReLU multipliers in either or both layers, and the shapes
    the kernel refuses."""
    torch = torch_cuda()
    from workloads import prelu_mult_neg
    n, h, w, c, cout = 3, 14, 14, 384, 96
    for case, (dsr, psr, dneg, pneg) in enumerate([((0, 4), (0, 6), False, False), ((3, 8), (4, 8), True, False),
                                                   ((3, 8), (4, 8), False, True), ((0, 5), (0, 5), True, True)]):
        D = make_dw_layer(7300 + case, n, h, w, c, 1, signed_x=True, act_window=(-128, 127), shift_range=dsr)
        Q = make_pw_layer(7310 + case, n, h, w, c, cout, act_window=(-128, 127), shift_range=psr, make_x=False)
        dn = prelu_mult_neg(7320 + case, D.mult) if dneg else None
        pn = prelu_mult_neg(7330 + case, Q.mult) if pneg else None
        mid = oracle.dw_conv(D.x, D.weight, 1, D.bias, D.mult, D.shift, -128, 127, mult_neg=dn)
        want = oracle.pw_conv(mid, Q.weight, Q.bias, Q.mult, Q.shift, -128, 127, mult_neg=pn)
        rqd = P.Requant(dev(D.bias), dev(D.mult), dev(D.shift), -128, 127, dev(dn) if dneg else None)
        rqp = P.Requant(dev(Q.bias), dev(Q.mult), dev(Q.shift), -128, 127, dev(pn) if pneg else None)
        y = P.prom_dw_pw_conv(dev(D.x), dev(D.weight), 1, rqd, dev(P.prom_pack_ternary(Q.weight)), cout, rqp)
        torch.cuda.synchronize()
        assert_same(y.cpu().numpy(), want, f"dw+pw case {case}")
    assert not P.prom_dw_pw_can_fuse(1, 8, 8, 24, 16, 1)     # c % 16 != 0
    assert not P.prom_dw_pw_can_fuse(1, 8, 8, 32, 336, 1)    # more than 320 output channels
    assert not P.prom_dw_pw_can_fuse(1, 8, 200, 32, 16, 1)   # three input rows are more than 256 pixels
    assert P.prom_dw_pw_can_fuse(128, 14, 14, 576, 96, 1) and P.prom_dw_pw_can_fuse(128, 7, 7, 960, 320, 1)
