"""The pointwise kernel for wide layers (k loop outermost over a 128-channel x 256-pixel workgroup
tile, plan field k_outer) against the CPU oracle, bit for bit: forced on shapes with ragged pixel
counts and channel counts off the tile sizes, with and without the skip connection (also in place),
shifts down to 0, the PReLU epilogue, and the shapes the library takes it for by itself."""
import numpy as np
import pytest

import oracle
from workloads import make_pw_layer
from gpu_util import run_pw, oracle_pw, assert_same, dev, requant_dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


WIDE_SHAPES = [
    # n, h, w, cin, cout: one and many k steps (odd and even counts), one ragged and several column
    # tiles of 128 channels, pixel counts below one row tile, ragged, and several row tiles
    (1, 1, 1, 64, 16), (3, 7, 7, 64, 400), (2, 14, 14, 192, 128), (1, 5, 13, 320, 144),
    (2, 9, 9, 512, 1024), (1, 14, 14, 1024, 512), (4, 7, 7, 2048, 272), (1, 31, 33, 128, 640),
    (1, 20, 13, 4096, 32),
]


@pytest.mark.parametrize("shape", WIDE_SHAPES)
@pytest.mark.parametrize("res", [False, True])
def test_wide_kernel_forced(P, shape, res):
    n, h, w, cin, cout = shape
    L = make_pw_layer(9000 + cin + 3 * cout, n, h, w, cin, cout, signed_x=True,
                      act_window=(-128, 127) if res else (-20, 90), with_residual=res, shift_range=(0, 9))
    L.x.reshape(-1)[::37] = -128
    got = run_pw(P, L, plan=P.PwPlan(k_outer=1))
    assert_same(got, oracle_pw(oracle, L), f"wide kernel {shape} res={res}")
    # the streaming kernel on the same layer
    assert_same(run_pw(P, L, plan=P.PwPlan(k_outer=-1)), got, f"streaming kernel {shape} res={res}")


def test_wide_kernel_is_the_library_choice_for_wide_layers(P):
    assert P.prom_pw_plan_query(128, 14, 14, 1024, 512)["k_outer"] == 1
    assert P.prom_pw_plan_query(128, 7, 7, 2048, 1024)["k_outer"] == 1
    assert P.prom_pw_plan_query(128, 14, 14, 64, 384)["k_outer"] == 0
    assert P.prom_pw_plan_query(128, 7, 7, 960, 160)["k_outer"] == 0
    assert P.prom_pw_plan_query(128, 14, 14, 512, 1024)["k_outer"] == 0
    L = make_pw_layer(9100, 6, 14, 14, 1024, 512, with_residual=True, act_window=(-128, 127))
    assert_same(run_pw(P, L), oracle_pw(oracle, L), "library choice 1024 -> 512")


def test_wide_kernel_plan_limits(P):
    torch = torch_cuda()
    L = make_pw_layer(9200, 1, 4, 4, 72, 32)     # cin % 64 != 0
    with pytest.raises(P.PromError) as e:
        run_pw(P, L, plan=P.PwPlan(k_outer=1))
    assert e.value.code == -1
    L = make_pw_layer(9201, 1, 4, 4, 64, 32)
    with pytest.raises(P.PromError) as e:      # combined with a streaming-kernel plan
        run_pw(P, L, plan=P.PwPlan(k_outer=1, tiles_per_wave=2))
    assert e.value.code == -1
    with pytest.raises(P.PromError) as e:
        run_pw(P, L, plan=P.PwPlan(k_outer=2))
    assert e.value.code == -1
    torch.cuda.synchronize()


def test_wide_kernel_residual_in_place_and_prelu(P):
    torch = torch_cuda()
    L = make_pw_layer(9300, 3, 9, 11, 256, 384, signed_x=True, with_residual=True, act_window=(-128, 127),
                      shift_range=(2, 8))
    xd, wp, rq = dev(L.x), dev(P.prom_pack_ternary(L.weight)), requant_dev(P, L)
    y = dev(L.residual).clone()
    P.prom_pw_conv_ex(xd, wp, L.cout, rq, y, y=y, plan=P.PwPlan(k_outer=1))
    torch.cuda.synchronize()
    assert_same(y.cpu().numpy(), oracle_pw(oracle, L), "residual in place")
    # PReLU: negative side with its own multiplier
    rng = np.random.default_rng(5)
    mult_neg = rng.integers(-(1 << 30), 1 << 30, size=L.cout, dtype=np.int64).astype(np.int32)
    rqp = P.Requant(dev(L.bias), dev(L.mult), dev(L.shift), -128, 127, dev(mult_neg))
    yp = P.prom_pw_conv_ex(xd, wp, L.cout, rqp, None, plan=P.PwPlan(k_outer=1))
    torch.cuda.synchronize()
    want = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, -128, 127, residual=None, mult_neg=mult_neg)
    assert_same(yp.cpu().numpy(), want, "PReLU epilogue")
