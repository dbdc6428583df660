"""Parity of the device weight quantisers with the oracle: codes, packed words and scales bit for
bit, on float32 weights of every MobileNetV2 pointwise and depthwise layer shape (Kaiming-normal
and a 'trained-like' variant with widely different row scales, dead channels and rounding ties),
and the quantised weights fed straight into the convolution kernels."""
import numpy as np
import pytest

import oracle
from workloads import (float_conv_weights, make_pw_layer, make_dw_layer, mobilenetv2_pointwise_layers,
                       mobilenetv2_depthwise_layers)
from gpu_util import assert_same, dev, requant_dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def _check_pw(P, w, tag):
    torch = torch_cuda()
    packed, scale, codes = P.prom_quantize_pw_absmean(dev(w), want_codes=True)
    torch.cuda.synchronize()
    q, s = oracle.quantize_pw_absmean(w)
    assert_same(codes.cpu().numpy(), q, f"{tag}: codes")
    assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32)), f"{tag}: scales"
    assert_same(packed.cpu().numpy(), P.prom_pack_ternary(q).reshape(-1), f"{tag}: packed words")


@pytest.mark.parametrize("kind", ["kaiming", "trained"])
def test_absmean_every_mobilenetv2_pointwise_shape(P, kind):
    seen = set()
    for i, s in enumerate(mobilenetv2_pointwise_layers()):
        if (s.cin, s.cout) in seen:
            continue
        seen.add((s.cin, s.cout))
        _check_pw(P, float_conv_weights(8000 + i, s.cout, s.cin, kind=kind), f"{kind} {s.cin}->{s.cout}")


def test_absmean_edge_shapes(P):
    for cout, cin in ((1, 1), (3, 5), (7, 16), (5, 17), (2, 1025), (130, 31), (1, 4096)):
        _check_pw(P, float_conv_weights(8100 + cin, cout, cin, kind="trained"), f"{cout}x{cin}")
    z = np.zeros((4, 40), dtype=np.float32)
    _check_pw(P, z, "all zero")


@pytest.mark.parametrize("kind", ["kaiming", "trained"])
def test_absmax_every_mobilenetv2_depthwise_shape(P, kind):
    torch = torch_cuda()
    for c in sorted({d.c for d in mobilenetv2_depthwise_layers()} | {1, 5, 257}):
        w = float_conv_weights(8200 + c, c, 9, kind=kind).reshape(c, 3, 3)
        wq, scale = P.prom_quantize_dw_absmax(dev(w))
        torch.cuda.synchronize()
        q, s = oracle.quantize_dw_absmax(w)
        assert_same(wq.cpu().numpy(), q, f"{kind} dw c={c}")
        assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32))


@pytest.mark.parametrize("kind", ["kaiming", "trained"])
def test_absmax_grouped_layers(P, kind):
    """Grouped 3x3 weights of the RegNetX / ResNeXt shapes (and ragged ones): codes and scales
    bit for bit, and the quantised layer runs through prom_gconv3x3."""
    torch = torch_cuda()
    for c, gs in ((32, 16), (160, 16), (128, 4), (256, 8), (1024, 32), (48, 24), (10, 5), (64, 64), (7, 1)):
        w = float_conv_weights(8300 + c + gs, c, 9 * gs, kind=kind).reshape(c, gs, 3, 3)
        wq, scale = P.prom_quantize_gconv_absmax(dev(w))
        torch.cuda.synchronize()
        q, s = oracle.quantize_gconv_absmax(w)
        assert_same(wq.cpu().numpy(), q, f"{kind} grouped c={c} gs={gs}")
        assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32))
    z, sz = P.prom_quantize_gconv_absmax(dev(np.zeros((8, 4, 3, 3), np.float32)))
    torch.cuda.synchronize()
    assert not z.cpu().numpy().any() and np.all(sz.cpu().numpy() == np.float32(127.0) / np.float32(1e-5))
    lib = P.load_library()
    st = torch.cuda.current_stream().cuda_stream
    w = dev(np.zeros((8, 3, 3, 3), np.float32))
    assert lib.prom_quantize_gconv_absmax(w.data_ptr(), 8, 3, 1e-5, z.data_ptr(), sz.data_ptr(), st) == -1


def test_quantised_weights_feed_the_convolutions(P):
    """float32 weights -> device quantisers -> prom_pw_conv / prom_dw_conv, against the oracle's
    quantisers followed by the oracle's convolutions."""
    torch = torch_cuda()
    L = make_pw_layer(8300, 2, 14, 14, 64, 384)
    w = float_conv_weights(8301, 384, 64)
    packed, _, _ = P.prom_quantize_pw_absmean(dev(w))
    y = P.prom_pw_conv(dev(L.x), packed, 384, requant_dev(P, L))
    q, _ = oracle.quantize_pw_absmean(w)
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), oracle.pw_conv(L.x, q, L.bias, L.mult, L.shift, L.act_min, L.act_max), "pw")
    D = make_dw_layer(8310, 2, 14, 14, 384, 1)
    wd = float_conv_weights(8311, 384, 9).reshape(384, 3, 3)
    wq, _ = P.prom_quantize_dw_absmax(dev(wd))
    y = P.prom_dw_conv(dev(D.x), wq, 1, requant_dev(P, D))
    qd, _ = oracle.quantize_dw_absmax(wd)
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), oracle.dw_conv(D.x, qd, 1, D.bias, D.mult, D.shift, D.act_min, D.act_max), "dw")


def test_quantiser_argument_errors(P):
    torch = torch_cuda()
    lib = P.load_library()
    w = torch.zeros((4, 16), dtype=torch.float32, device="cuda")
    out = torch.zeros(64, dtype=torch.uint8, device="cuda")
    sc = torch.zeros(4, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    assert lib.prom_quantize_pw_absmean(w.data_ptr(), 4, 16, 1e-5, out.data_ptr(), 8, None, sc.data_ptr(), st) == -4
    assert lib.prom_quantize_pw_absmean(w.data_ptr(), 4, 16, 0.0, out.data_ptr(), 64, None, sc.data_ptr(), st) == -1
    assert lib.prom_quantize_pw_absmean(None, 4, 16, 1e-5, out.data_ptr(), 64, None, sc.data_ptr(), st) == -1
    assert lib.prom_quantize_dw_absmax(w.data_ptr(), 0, 1e-5, out.data_ptr(), sc.data_ptr(), st) == -1


def test_activation_absmax_per_sample(P):
    """The paper's dynamic activation quantiser: one absmax scale per batch element.  Codes and
    scales bit for bit, for images of very different magnitude, sizes off the 4-element vector
    width, an all-zero image and one below eps."""
    torch = torch_cuda()
    rng = np.random.default_rng(8400)
    for shape in ((6, 14, 14, 384), (3, 5, 7, 3), (1, 56, 56, 144), (5, 1), (2, 1025), (64, 7, 7, 160)):
        x = rng.standard_normal(shape).astype(np.float32)
        for i in range(shape[0]):
            x[i] *= np.float32(10.0 ** rng.integers(-4, 5))
        if shape[0] > 2:
            x[1] = 0.0
            x[2] *= np.float32(1e-9)
        q, scale = P.prom_quantize_activation_absmax(dev(x))
        torch.cuda.synchronize()
        want, s = oracle.quantize_activation_absmax(x)
        assert_same(q.cpu().numpy(), want, f"activation codes {shape}")
        assert np.array_equal(scale.cpu().numpy().view(np.uint32), s.view(np.uint32)), f"scales {shape}"
    # twice in a row into the same buffers: the scratch use of `scale` leaves nothing behind
    x = rng.standard_normal((4, 28, 28, 32)).astype(np.float32)
    xd = dev(x)
    q, scale = P.prom_quantize_activation_absmax(xd)
    q2, scale2 = P.prom_quantize_activation_absmax(dev(x * np.float32(0.5)), q=q, scale=scale)
    torch.cuda.synchronize()
    want, s = oracle.quantize_activation_absmax(x * np.float32(0.5))
    assert_same(q2.cpu().numpy(), want, "second call") and np.array_equal(scale2.cpu().numpy(), s)
