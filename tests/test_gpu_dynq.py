"""GPU parity of prom_pw_conv_dynq (pointwise layer with the dynamic per-image activation scale,
Section 3.1, Eq. 6-7) against the oracle, bit for bit: codes, per-image maxima and scales.  Both
sides take every float32 operation in the same order, so the comparison is exact."""
import numpy as np
import pytest

import oracle
from workloads import make_pw_layer
from gpu_util import torch_cuda, dev, assert_same

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def factors(seed, n, cout):
    rng = np.random.default_rng(seed)
    x_step = (rng.uniform(0.002, 0.05, n) * 2.0 ** rng.integers(-3, 4, n)).astype(np.float32)
    w_scale = rng.uniform(0.01, 0.2, cout).astype(np.float32)
    bias = rng.normal(0, 0.5, cout).astype(np.float32)
    return x_step, w_scale, bias


def run_case(P, L, x_step, w_scale, bias, relu, eps=1e-5):
    torch = torch_cuda()
    q, amax, scale = P.prom_pw_conv_dynq(dev(L.x), dev(P.prom_pack_ternary(L.weight)), L.cout, dev(x_step),
                                         dev(w_scale), dev(bias) if bias is not None else None, relu, eps)
    torch.cuda.synchronize()
    wq, wamax, wscale = oracle.pw_conv_dynamic_quant(L.x, L.weight, x_step, w_scale, bias, relu, eps)
    what = f"{L.n}x{L.h}x{L.w} {L.cin}->{L.cout} relu={relu} bias={bias is not None}"
    assert np.array_equal(amax.cpu().numpy(), wamax), f"{what}: per-image maxima differ"
    assert np.array_equal(scale.cpu().numpy(), wscale), f"{what}: scales differ"
    assert_same(q.cpu().numpy(), wq, what)


# (n, hw, cin, cout): ragged pixel counts, images that straddle 16-pixel tiles (7x7, 5x5, 1x1),
# ragged k steps, one to three channel chunks, widths that are not multiples of 64
SHAPES = [(3, 7, 16, 16), (5, 5, 32, 48), (2, 14, 64, 384), (4, 9, 96, 144), (17, 1, 160, 80),
          (2, 28, 144, 32), (3, 7, 576, 160), (2, 7, 960, 320), (1, 10, 1024, 64), (8, 56, 24, 144), (3, 6, 40, 16), (2, 5, 100, 32),
          (2, 11, 320, 1280)]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("relu", [False, True])
def test_dynq_matches_the_oracle(P, shape, relu):
    n, hw, cin, cout = shape
    L = make_pw_layer(4200 + cin + cout, n, hw, hw, cin, cout, signed_x=True)
    x_step, w_scale, bias = factors(cin + cout, n, cout)
    run_case(P, L, x_step, w_scale, bias if relu or cin % 32 == 0 else None, relu)


def test_dynq_zero_image_and_tiny_values(P):
    L = make_pw_layer(4300, 4, 6, 6, 32, 32, signed_x=True)
    L.x[1] = 0                                   # an image of zeros: maximum 0, scale 127 / eps
    x_step, w_scale, _ = factors(9, 4, 32)
    x_step[2] = np.float32(1e-9)                 # an image whose values stay below eps
    run_case(P, L, x_step, w_scale, None, False)
    run_case(P, L, x_step, w_scale, None, True, eps=1e-3)


def test_dynq_twice_in_a_row_and_limits(P):
    torch = torch_cuda()
    L = make_pw_layer(4400, 2, 8, 8, 48, 64, signed_x=True)
    x_step, w_scale, bias = factors(10, 2, 64)
    for _ in range(2):   # the maxima are cleared by the call itself
        run_case(P, L, x_step, w_scale, bias, False)
    x = dev(L.x)
    wp = dev(P.prom_pack_ternary(L.weight))
    with pytest.raises(P.PromError):             # cin % 4 != 0
        P.prom_pw_conv_dynq(x[..., :42].contiguous(), wp, 64, dev(x_step), dev(w_scale))
    with pytest.raises(P.PromError):             # eps <= 0
        P.prom_pw_conv_dynq(x, wp, 64, dev(x_step), dev(w_scale), eps=0.0)
    torch.cuda.synchronize()
