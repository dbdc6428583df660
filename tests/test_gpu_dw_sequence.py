"""prom_dw_conv_sequence: several depthwise layers with one host call.  Independent layers share
one launch, dependent ones are launched one after the other; either way every output equals the
oracle's (paper Section 3.1 "Depthwise Convolutions": 8-bit 3x3 depthwise convolution)."""
import numpy as np
import pytest

import oracle
from workloads import make_dw_layer, mobilenetv2_depthwise_layers
from gpu_util import assert_same, dev, requant_dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def want_of(D, stride, mult_neg=None):
    return oracle.dw_conv(D.x, D.weight, stride, D.bias, D.mult, D.shift, D.act_min, D.act_max, mult_neg=mult_neg)


def test_all_mobilenetv2_depthwise_layers_in_one_call(P):
    torch = torch_cuda()
    layers, wants, names = [], [], []
    for i, d in enumerate(mobilenetv2_depthwise_layers()):
        D = make_dw_layer(7100 + i, 3, d.hw_in, d.hw_in, d.c, d.stride, signed_x=(i % 2 == 1),
                          act_window=(-128, 127) if i % 2 else (0, 127))
        ho = (d.hw_in - 1) // d.stride + 1
        y = torch.full((3, ho, ho, d.c), -77, dtype=torch.int8, device="cuda")
        layers.append((dev(D.x), dev(D.weight), d.stride, requant_dev(P, D), y))
        wants.append(want_of(D, d.stride))
        names.append(d.name)
    seq = P.DwSequence(layers)
    for run in range(2):
        seq.run()
        torch.cuda.synchronize()
        for name, want, lay in zip(names, wants, layers):
            assert_same(lay[4].cpu().numpy(), want, f"run {run}, {name}")
            lay[4].fill_(-77)


def test_mixed_shapes_ragged_and_dependent_layers(P):
    torch = torch_cuda()
    # ragged widths and heights, stride 1 with fewer than 8 rows, stride 2, channels not a multiple
    # of 4 (the one-thread-per-output kernel: launched alone), and a layer that reads the one before
    shapes = [(2, 9, 13, 24, 1), (1, 5, 7, 40, 1), (3, 11, 6, 16, 2), (2, 8, 8, 6, 1), (2, 17, 17, 32, 1)]
    inputs, layers = [], []
    for i, (n, h, w, c, s) in enumerate(shapes):
        D = make_dw_layer(7200 + i, n, h, w, c, s, signed_x=True, act_window=(-128, 127))
        y = torch.full((n, (h - 1) // s + 1, (w - 1) // s + 1, c), -77, dtype=torch.int8, device="cuda")
        layers.append((dev(D.x), dev(D.weight), s, requant_dev(P, D), y))
        inputs.append(D)
    # a sixth layer whose input is the fifth layer's output
    D6 = make_dw_layer(7300, 2, 17, 17, 32, 2, signed_x=True, act_window=(-128, 127))
    y6 = torch.full((2, 9, 9, 32), -77, dtype=torch.int8, device="cuda")
    layers.append((layers[4][4], dev(D6.weight), 2, requant_dev(P, D6), y6))
    P.prom_dw_conv_sequence(layers)
    torch.cuda.synchronize()
    mids = []
    for (n, h, w, c, s), D, lay in zip(shapes, inputs, layers):
        want = want_of(D, s)
        mids.append(want)
        assert_same(lay[4].cpu().numpy(), want, f"{n}x{h}x{w}x{c} stride {s}")
    want6 = oracle.dw_conv(mids[4], D6.weight, 2, D6.bias, D6.mult, D6.shift, -128, 127)
    assert_same(y6.cpu().numpy(), want6, "layer fed by the layer before it")


def test_sequence_reports_the_offending_layer_and_enqueues_nothing(P):
    torch = torch_cuda()
    D = make_dw_layer(7400, 1, 8, 8, 16, 1)
    x, w, rq = dev(D.x), dev(D.weight), requant_dev(P, D)
    y0 = torch.full((1, 8, 8, 16), -77, dtype=torch.int8, device="cuda")
    with pytest.raises(P.PromError) as e:
        P.prom_dw_conv_sequence([(x, w, 1, rq, y0), (x, w, 3, rq, torch.empty_like(y0))])   # stride 3
    assert "layer 1" in str(e.value)
    torch.cuda.synchronize()
    assert int((y0 != -77).sum()) == 0
    with pytest.raises(P.PromError):                                                        # y aliases x
        P.prom_dw_conv_sequence([(x, w, 1, rq, x)])
    P.prom_dw_conv_sequence([])                                                             # empty: nothing to do
    torch.cuda.synchronize()


def test_batches_that_are_multiples_of_eight_take_the_image_order(P):
    """With a multiple of 8 images a layer's workgroups are laid out so that 8 consecutive ones are the
    same place in 8 images (alone: a flat grid; in a shared launch: per member, with the members'
    ranges padded to multiples of 8); mixed here with batches that keep the plain order."""
    torch = torch_cuda()
    shapes = [(8, 14, 14, 96, 1), (16, 7, 7, 160, 1), (3, 9, 13, 24, 1), (8, 28, 28, 32, 2), (24, 5, 6, 64, 1),
              (8, 17, 11, 48, 2), (5, 8, 8, 16, 1), (16, 12, 12, 40, 1)]
    layers, wants = [], []
    for i, (n, h, w, c, s) in enumerate(shapes):
        D = make_dw_layer(7500 + i, n, h, w, c, s, signed_x=True, act_window=(-128, 127))
        ho, wo = (h - 1) // s + 1, (w - 1) // s + 1
        y = torch.full((n, ho, wo, c), -77, dtype=torch.int8, device="cuda")
        layers.append((dev(D.x), dev(D.weight), s, requant_dev(P, D), y))
        wants.append(want_of(D, s))
        # alone
        got = P.prom_dw_conv(layers[-1][0], layers[-1][1], s, layers[-1][3])
        torch.cuda.synchronize()
        assert_same(got.cpu().numpy(), wants[-1], f"alone {shapes[i]}")
    P.prom_dw_conv_sequence(layers)
    torch.cuda.synchronize()
    for shape, want, lay in zip(shapes, wants, layers):
        assert_same(lay[4].cpu().numpy(), want, f"in one call {shape}")
