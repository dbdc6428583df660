"""Parity of prom_gconv3x3 (grouped 3x3 convolution, int8) against the CPU oracle: bit-exact."""
import numpy as np
import pytest

import oracle
from workloads import make_gconv_layer, prelu_mult_neg
from gpu_util import assert_same, dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def _run(P, G, window=None, mneg=None, offset_params=False, use_frag=False):
    torch = torch_cuda()
    lo, hi = window if window is not None else (G.act_min, G.act_max)
    if offset_params:  # parameter arrays that are not 16-byte aligned
        pad = lambda a: dev(np.concatenate([np.zeros(1, a.dtype), a]))[1:]
    else:
        pad = dev
    rq = P.Requant(pad(G.bias), pad(G.mult), pad(G.shift), lo, hi, None if mneg is None else pad(mneg))
    frag = dev(P.prom_gconv_pack(G.weight)) if use_frag else None
    y = P.prom_gconv3x3(dev(G.x), dev(G.weight), G.stride, rq, w_frag=frag)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def _want(G, window=None, mneg=None):
    lo, hi = window if window is not None else (G.act_min, G.act_max)
    return oracle.gconv3x3(G.x, G.weight, G.stride, G.bias, G.mult, G.shift, lo, hi, mult_neg=mneg)


SHAPES = [
    # n, h, w, c, gs, stride: every chunking of the tiled kernel (gs 4, 8, 16 in one chunk; 12, 24,
    # 32, 40, 48, 64 in several), one group = dense conv, odd sizes, 1..3 rows left over in the
    # row groups of 4, one pixel, group sizes and channel counts of the one-thread-per-output kernel
    (2, 9, 11, 16, 4, 1), (2, 9, 11, 16, 4, 2), (1, 14, 14, 64, 8, 1), (2, 7, 7, 64, 8, 2),
    (2, 13, 10, 64, 16, 1), (1, 28, 28, 128, 16, 2), (1, 6, 5, 24, 12, 1), (1, 7, 9, 48, 24, 1),
    (2, 5, 6, 48, 24, 2), (1, 9, 9, 64, 32, 1), (1, 10, 7, 80, 40, 2), (1, 8, 8, 96, 48, 1),
    (1, 5, 5, 128, 64, 2), (1, 6, 6, 32, 32, 1), (1, 1, 1, 16, 8, 1), (3, 2, 2, 8, 4, 2),
    (2, 5, 4, 6, 3, 1), (1, 7, 3, 10, 5, 2), (2, 4, 4, 6, 2, 1), (1, 5, 5, 12, 1, 1), (1, 4, 6, 7, 7, 2),
    (4, 56, 56, 96, 16, 1), (4, 56, 56, 96, 16, 2), (2, 28, 28, 192, 48, 1),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_gconv_shapes(P, shape):
    n, h, w, c, gs, stride = shape
    G = make_gconv_layer(15000 + h * 31 + c + gs + stride, n, h, w, c, gs, stride, signed_x=True,
                         act_window=(-128, 127), shift_range=(8, 17))
    G.x.reshape(-1)[::37] = -128
    want = _want(G)
    assert_same(_run(P, G), want, f"gconv {shape}")
    if P.prom_gconv_frag_size(c, gs):  # the matrix-core kernel with weights prepared by prom_gconv_pack
        assert_same(_run(P, G, use_frag=True), want, f"gconv {shape} prepared weights")


@pytest.mark.parametrize("shape", [(2, 9, 11, 32, 8, 1), (2, 9, 11, 48, 24, 2), (1, 6, 6, 10, 5, 1)])
def test_gconv_prelu_windows_shifts_and_unaligned_parameters(P, shape):
    n, h, w, c, gs, stride = shape
    G = make_gconv_layer(15500 + c + gs, n, h, w, c, gs, stride, signed_x=True, shift_range=(0, 31))
    mneg = prelu_mult_neg(15500 + c, G.mult)
    mneg[::3] = -(1 << 31)
    for window in ((-128, 127), (0, 127), (-5, 9)):
        assert_same(_run(P, G, window), _want(G, window), f"plain {shape} {window}")
        assert_same(_run(P, G, window, mneg), _want(G, window, mneg), f"prelu {shape} {window}")
        if P.prom_gconv_frag_size(c, gs):
            assert_same(_run(P, G, window, mneg, use_frag=True), _want(G, window, mneg), f"prelu frag {shape}")
    assert_same(_run(P, G, None, mneg, offset_params=True), _want(G, None, mneg), f"unaligned {shape}")


def test_gconv_group_size_one_is_the_depthwise_layer(P):
    torch = torch_cuda()
    G = make_gconv_layer(15600, 2, 14, 14, 96, 1, 2, signed_x=True, act_window=(-128, 127))
    rq = P.Requant(dev(G.bias), dev(G.mult), dev(G.shift), -128, 127)
    a = P.prom_gconv3x3(dev(G.x), dev(G.weight), 2, rq)
    b = P.prom_dw_conv(dev(G.x), dev(G.weight.reshape(3, 3, 96)), 2, rq)
    torch.cuda.synchronize()
    assert_same(a.cpu().numpy(), b.cpu().numpy(), "group size 1")
    assert_same(a.cpu().numpy(), _want(G), "group size 1 vs oracle")


def test_gconv_argument_errors(P):
    G = make_gconv_layer(15700, 1, 4, 4, 16, 4)
    rq = P.Requant(dev(G.bias), dev(G.mult), dev(G.shift), 0, 127)
    x, w = dev(G.x), dev(G.weight)
    with pytest.raises(P.PromError) as e:
        P.prom_gconv3x3(x, dev(np.zeros((3, 3, 16, 3), np.int8)), 1, rq)   # 16 % 3 != 0
    assert e.value.code == -1
    with pytest.raises(P.PromError) as e:
        P.prom_gconv3x3(x, w, 3, rq)
    assert e.value.code == -1
    with pytest.raises(P.PromError) as e:
        P.prom_gconv3x3(x, w, 1, rq, y=x)                                    # output over input
    assert e.value.code == -3
    G5 = make_gconv_layer(15701, 1, 4, 4, 10, 5)                             # no prepared form for gs = 5
    with pytest.raises(P.PromError) as e:
        P.prom_gconv_pack(G5.weight)
    assert e.value.code == -2
    with pytest.raises(P.PromError) as e:
        P.prom_gconv3x3(dev(G5.x), dev(G5.weight), 1,
                        P.Requant(dev(G5.bias), dev(G5.mult), dev(G5.shift), 0, 127), w_frag=w)
    assert e.value.code == -1


def test_gconv_full_size_layer_every_output(P):
    """A layer of RegNetX-400MF's size at batch 32 (28x28, 160 channels in groups of 16), both
    strides, every output, three runs."""
    torch = torch_cuda()
    for stride in (1, 2):
        G = make_gconv_layer(15800 + stride, 32, 28, 28, 160, 16, stride)
        want = dev(_want(G))
        x, w, frag = dev(G.x), dev(G.weight), dev(P.prom_gconv_pack(G.weight))
        rq = P.Requant(dev(G.bias), dev(G.mult), dev(G.shift), G.act_min, G.act_max)
        for run in range(3):
            y = P.prom_gconv3x3(x, w, stride, rq, w_frag=frag if run else None)
            torch.cuda.synchronize()
            bad = int((y != want).sum())
            assert bad == 0, f"stride {stride}, run {run}: {bad} outputs differ"


def _seq_entry(P, G, window=(-128, 127), mneg=None, use_frag=False, x=None):
    torch = torch_cuda()
    lo, hi = window
    rq = P.Requant(dev(G.bias), dev(G.mult), dev(G.shift), lo, hi, None if mneg is None else dev(mneg))
    n, h, w, c = G.x.shape
    ho, wo = (h - 1) // G.stride + 1, (w - 1) // G.stride + 1
    y = torch.full((n, ho, wo, c), 77, dtype=torch.int8, device="cuda:0")
    frag = dev(P.prom_gconv_pack(G.weight)) if use_frag else None
    return (dev(G.x) if x is None else x, dev(G.weight), G.stride, rq, y, frag)


def test_gconv_sequence_of_independent_layers(P):
    """Layers of every kernel in one call: the matrix-core ones share launches (members of different
    shapes, band heights, strides, epilogue forms, with and without prepared weights), the others are
    launched one by one; every output equals the oracle's."""
    torch = torch_cuda()
    specs = [  # n, h, w, c, gs, stride, shift range, prelu, prepared weights
        (4, 56, 56, 96, 16, 1, (8, 17), False, True), (2, 9, 11, 16, 4, 2, (0, 31), False, False),
        (3, 14, 14, 64, 8, 1, (8, 17), True, True), (2, 7, 7, 128, 16, 1, (1, 12), False, True),
        (1, 28, 28, 40, 4, 2, (8, 17), False, False), (5, 7, 7, 384, 16, 1, (8, 17), False, True),
        (1, 9, 9, 64, 32, 1, (8, 17), False, True), (2, 5, 5, 128, 64, 2, (0, 31), True, False),
        (1, 6, 5, 24, 12, 1, (8, 17), False, False), (1, 5, 5, 12, 1, 1, (8, 17), False, False),
        (2, 13, 10, 64, 16, 1, (8, 17), False, True),
    ]
    entries, wants = [], []
    for i, (n, h, w, c, gs, s, sr, prelu, frag) in enumerate(specs):
        G = make_gconv_layer(15700 + i, n, h, w, c, gs, s, signed_x=True, act_window=(-128, 127), shift_range=sr)
        mneg = prelu_mult_neg(15700 + i, G.mult) if prelu else None
        entries.append(_seq_entry(P, G, mneg=mneg, use_frag=frag))
        wants.append(_want(G, (-128, 127), mneg))
    P.prom_gconv3x3_sequence(entries)
    torch.cuda.synchronize()
    for i, (e, want) in enumerate(zip(entries, wants)):
        assert_same(e[4].cpu().numpy(), want, f"sequence member {i} {specs[i]}")
    # the same array again, and through a prebuilt sequence object
    seq = P.GconvSequence(entries)
    for e in entries:
        e[4].fill_(55)
    seq.run()
    torch.cuda.synchronize()
    for i, (e, want) in enumerate(zip(entries, wants)):
        assert_same(e[4].cpu().numpy(), want, f"prebuilt sequence member {i}")


def test_gconv_sequence_keeps_the_order_of_dependent_layers(P):
    """A layer that reads what an earlier one writes does not share its launch: the result is that
    of running the layers one after the other."""
    torch = torch_cuda()
    G1 = make_gconv_layer(15800, 2, 14, 14, 64, 16, 1, signed_x=True, act_window=(-128, 127))
    G2 = make_gconv_layer(15801, 2, 14, 14, 64, 8, 2, signed_x=True, act_window=(-128, 127))
    G3 = make_gconv_layer(15802, 2, 14, 14, 64, 4, 1, signed_x=True, act_window=(-128, 127))
    e1 = _seq_entry(P, G1, use_frag=True)
    e2 = _seq_entry(P, G2, x=e1[4])           # reads the first layer's output
    e3 = _seq_entry(P, G3, use_frag=True)     # independent of both
    P.prom_gconv3x3_sequence([e1, e2, e3])
    torch.cuda.synchronize()
    y1 = _want(G1, (-128, 127))
    assert_same(e1[4].cpu().numpy(), y1, "first layer")
    y2 = oracle.gconv3x3(y1, G2.weight, G2.stride, G2.bias, G2.mult, G2.shift, -128, 127)
    assert_same(e2[4].cpu().numpy(), y2, "second layer on the first one's output")
    assert_same(e3[4].cpu().numpy(), _want(G3, (-128, 127)), "third layer")


def test_gconv_sequence_errors_and_empty(P):
    torch = torch_cuda()
    P.prom_gconv3x3_sequence([])
    G1 = make_gconv_layer(15900, 1, 6, 6, 16, 4, 1)
    G2 = make_gconv_layer(15901, 1, 6, 6, 16, 4, 1)
    e1 = _seq_entry(P, G1)
    e2 = list(_seq_entry(P, G2))
    e2[2] = 3  # no such stride
    with pytest.raises(P.PromError) as err:
        P.prom_gconv3x3_sequence([e1, tuple(e2)])
    assert err.value.code == -1 and "layer 1" in str(err.value)
    torch.cuda.synchronize()
    assert bool((e1[4] == 77).all()), "nothing is enqueued when a layer is refused"
    # an output that overlaps its own input
    e3 = list(_seq_entry(P, G1))
    e3[4] = e3[0]
    with pytest.raises(P.PromError) as err:
        P.prom_gconv3x3_sequence([tuple(e3)])
    assert err.value.code == -3


@pytest.mark.parametrize("family,batch", [("regnetx_400mf", 128), ("resnext50_32x4d", 128),
                                          ("regnetx_400mf", 256), ("regnetx_400mf", 48)])
def test_gconv_sequence_at_benchmark_size_equals_layer_by_layer(P, family, batch):
    """The shared launches of the benchmark's configuration (batch 128, every grouped 3x3 layer of the
    network in one call: workgroup shares, XCD-aware order and padding as timed there) give, byte for
    byte, what the layers give one by one (the single-layer path is checked against the oracle above,
    one full-size layer on every output).  Also at batch 256, where layers hand workgroups on to the
    layer that would end last, and at a batch that is no multiple of 64."""
    torch = torch_cuda()
    from workloads import regnetx_400mf_grouped_layers, resnext50_32x4d_grouped_layers
    shapes = regnetx_400mf_grouped_layers() if family == "regnetx_400mf" else resnext50_32x4d_grouped_layers()
    entries, singles = [], []
    for i, g in enumerate(shapes):
        G = make_gconv_layer(16000 + i, 1, 4, 4, g.c, g.gs, g.stride, shift_range=(8, 17) if i % 3 else (0, 31))
        ho = (g.hw_in - 1) // g.stride + 1
        x = torch.randint(-128, 128, (batch, g.hw_in, g.hw_in, g.c), dtype=torch.int8, device="cuda:0")
        rq = P.Requant(dev(G.bias), dev(G.mult), dev(G.shift), -128, 127)
        w = dev(G.weight)
        frag = dev(P.prom_gconv_pack(G.weight))
        y = torch.full((batch, ho, ho, g.c), 77, dtype=torch.int8, device="cuda:0")
        entries.append((x, w, g.stride, rq, y, frag))
        singles.append(P.prom_gconv3x3(x, w, g.stride, rq, w_frag=frag))
    P.prom_gconv3x3_sequence(entries)
    torch.cuda.synchronize()
    for i, (e, want) in enumerate(zip(entries, singles)):
        assert torch.equal(e[4], want), f"{family} layer {i} {shapes[i]}"
    # one layer of each shape against the oracle on a sample of images
    seen = set()
    for i, g in enumerate(shapes):
        key = (g.hw_in, g.c, g.gs, g.stride)
        if key in seen or g.hw_in > 28:
            continue
        seen.add(key)
        G = make_gconv_layer(16000 + i, 1, 4, 4, g.c, g.gs, g.stride, shift_range=(8, 17) if i % 3 else (0, 31))
        xs = entries[i][0][:2].cpu().numpy()
        want = oracle.gconv3x3(xs, G.weight, g.stride, G.bias, G.mult, G.shift, -128, 127)
        assert_same(entries[i][4][:2].cpu().numpy(), want, f"{family} layer {i} against the oracle")


def test_gconv_matrix_core_kernels_on_random_shapes(P):
    """Seeded random shapes for the two matrix-core kernels: odd sizes down to one pixel, channel counts
    that leave a partial block of 64, several images per unit of work, both strides, all three epilogue
    forms, prepared and unprepared weights; and the same layers again through one sequence call."""
    torch = torch_cuda()
    rng = np.random.default_rng(20250511)
    entries, wants = [], []
    for case in range(48):
        gs = int(rng.choice([4, 8, 16, 32, 64]))
        c = gs * int(rng.integers(1, max(2, 200 // gs)))
        n, h, w = int(rng.integers(1, 10)), int(rng.integers(1, 21)), int(rng.integers(1, 21))
        stride = int(rng.integers(1, 3))
        prelu = bool(rng.integers(0, 2))
        window = [(-128, 127), (0, 127), (-7, 19)][int(rng.integers(0, 3))]
        sr = (8, 17) if rng.integers(0, 2) else (0, 31)
        G = make_gconv_layer(17000 + case, n, h, w, c, gs, stride, signed_x=True, act_window=window, shift_range=sr)
        mneg = prelu_mult_neg(17000 + case, G.mult) if prelu else None
        use_frag = bool(rng.integers(0, 2))
        want = _want(G, window, mneg)
        got = _run(P, G, window, mneg, use_frag=use_frag)
        assert_same(got, want, f"case {case}: n={n} h={h} w={w} c={c} gs={gs} s={stride} prelu={prelu} {window} frag={use_frag}")
        entries.append(_seq_entry(P, G, window, mneg, use_frag))
        wants.append(want)
    P.prom_gconv3x3_sequence(entries)
    torch.cuda.synchronize()
    for case, (e, want) in enumerate(zip(entries, wants)):
        assert_same(e[4].cpu().numpy(), want, f"sequence, case {case}")
