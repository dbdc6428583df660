"""Largest sizes: tensors at and beyond the 2 GiB limit of the kernels' 32-bit byte offsets.
Inputs are seeded and generated on the device (they would not fit a host array comfortably);
blocks of pixels / whole images at the start, at the end and in between are copied back and
checked against the oracle, which computes each output from its own inputs only."""
import numpy as np
import pytest

import oracle
from workloads import make_pw_layer, make_dw_layer, make_gconv_layer
from gpu_util import assert_same, dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def _device_bytes(torch, shape, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randint(-128, 128, shape, dtype=torch.int8, device="cuda", generator=g)


@pytest.mark.parametrize("n,fast", [(100, True), (104, False)])
def test_pw_at_and_beyond_the_streaming_limit(P, n, fast):
    """16 -> 96 channels on n x 470 x 470 pixels: 2.12 GB of output with n = 100 (just inside what
    the streaming kernel addresses), 2.21 GB with n = 104 (the generic kernel takes over)."""
    torch = torch_cuda()
    h = w = 470
    cin, cout = 16, 96
    m = n * h * w
    limit = (1 << 31) - (1 << 16) - (1 << 24)
    assert ((m + 4096) * cout < limit) == fast
    L = make_pw_layer(17000 + n, 1, 1, 1, cin, cout, signed_x=True, act_window=(-128, 127), shift_range=(2, 5))
    x = _device_bytes(torch, (n, h, w, cin), 17000 + n)
    rq = P.Requant(dev(L.bias), dev(L.mult), dev(L.shift), -128, 127)
    y = torch.full((n, h, w, cout), 77, dtype=torch.int8, device="cuda")
    P.prom_pw_conv(x, dev(P.prom_pack_ternary(L.weight)), cout, rq, None, y)
    torch.cuda.synchronize()
    xf, yf = x.view(m, cin), y.view(m, cout)
    rng = np.random.default_rng(n)
    starts = [0, m - 4096, m - 5000, (1 << 31) // cout - 2048] + [int(s) for s in rng.integers(0, m - 4096, 8)]
    for s in starts:
        s = max(0, min(s, m - 4096))
        xs = xf[s:s + 4096].cpu().numpy().reshape(1, 1, 4096, cin)
        want = oracle.pw_conv(xs, L.weight, L.bias, L.mult, L.shift, -128, 127).reshape(4096, cout)
        assert_same(yf[s:s + 4096].cpu().numpy(), want, f"pixels {s}..{s + 4095} of {m}")


def test_dw_tensor_beyond_2_gib(P):
    """20000 images of 28x28x144 (2.26 GB): the kernel addresses image by image."""
    torch = torch_cuda()
    n, hw, c = 20000, 28, 144
    D = make_dw_layer(17100, 1, 3, 3, c, 1, signed_x=True, act_window=(-128, 127))
    x = _device_bytes(torch, (n, hw, hw, c), 17100)
    rq = P.Requant(dev(D.bias), dev(D.mult), dev(D.shift), -128, 127)
    for stride in (1, 2):
        y = P.prom_dw_conv(x, dev(D.weight), stride, rq)
        torch.cuda.synchronize()
        for i in (0, 1, 9510, 9511, n - 2, n - 1):
            want = oracle.dw_conv(x[i:i + 1].cpu().numpy(), D.weight, stride, D.bias, D.mult, D.shift, -128, 127)
            assert_same(y[i:i + 1].cpu().numpy(), want, f"stride {stride} image {i}")
        del y


@pytest.mark.parametrize("n,mfma", [(18000, True), (20000, False)])
def test_gconv_at_and_beyond_2_gib(P, n, mfma):
    """28x28x144 in groups of 16: 2.03 GB with 18000 images (the matrix-core kernel, offsets up to
    its limit), 2.26 GB with 20000 (the per-image vector-ALU kernel takes over)."""
    torch = torch_cuda()
    hw, c, gs = 28, 144, 16
    assert (n * hw * hw * c < (1 << 31) - (1 << 24)) == mfma
    G = make_gconv_layer(17200, 1, 3, 3, c, gs, 1, signed_x=True, act_window=(-128, 127))
    x = _device_bytes(torch, (n, hw, hw, c), 17200 + n)
    rq = P.Requant(dev(G.bias), dev(G.mult), dev(G.shift), -128, 127)
    frag = dev(P.prom_gconv_pack(G.weight))
    y = P.prom_gconv3x3(x, dev(G.weight), 1, rq, w_frag=frag)
    torch.cuda.synchronize()
    for i in (0, 1, n // 2, n - 2, n - 1):
        want = oracle.gconv3x3(x[i:i + 1].cpu().numpy(), G.weight, 1, G.bias, G.mult, G.shift, -128, 127)
        assert_same(y[i:i + 1].cpu().numpy(), want, f"image {i} of {n}")


def test_requant_check_reports_the_first_bad_channel(P):
    """prom_requant_check copies the parameter arrays back and checks the documented preconditions:
    mult in (0, 2^31), shift in [0, 31], |bias| < 2^29, 128 * cin + |bias| < 2^30."""
    import torch
    from workloads import make_pw_layer
    from gpu_util import dev
    L = make_pw_layer(9900, 1, 2, 2, 64, 48)
    good = P.Requant(dev(L.bias), dev(L.mult), dev(L.shift), 0, 127)
    assert P.prom_requant_check(good, 64) == -1
    for what, arr, ch, val in (("mult", "mult", 5, 0), ("mult", "mult", 7, -3), ("shift", "shift", 11, 32),
                               ("shift", "shift", 2, -1), ("bias", "bias", 40, 1 << 29), ("bias", "bias", 41, -(1 << 29))):
        a = {"bias": L.bias.copy(), "mult": L.mult.copy(), "shift": L.shift.copy()}
        a[arr][ch] = val
        rq = P.Requant(dev(a["bias"]), dev(a["mult"]), dev(a["shift"]), 0, 127)
        assert P.prom_requant_check(rq, 64) == ch, (what, val)
    # the accumulator bound: a bias just below 2^29 is fine for few input channels, not for 2^22 of them
    b = L.bias.copy()
    b[3] = (1 << 29) - 1
    rq = P.Requant(dev(b), dev(L.mult), dev(L.shift), 0, 127)
    assert P.prom_requant_check(rq, 64) == -1
    assert P.prom_requant_check(rq, (1 << 22) + 1) == 3  # 128 * (2^22 + 1) + 2^29 - 1 >= 2^30
    torch.cuda.synchronize()
