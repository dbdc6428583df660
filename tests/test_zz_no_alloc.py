"""prom_block_noalloc (the block for callers that cannot allocate: its intermediates live in a
fixed array inside the library's device image) against prom_block with a caller workspace and
against the CPU oracle, bit for bit, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

import oracle
from workloads import make_block
from gpu_util import assert_same, dev, requant_dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def _run_both(P, B):
    torch = torch_cuda()
    e, d, p = B.expand, B.dw, B.project
    rqs = [requant_dev(P, l) for l in (e, d, p)]
    we, wd, wp = dev(P.prom_pack_ternary(e.weight)), dev(d.weight), dev(P.prom_pack_ternary(p.weight))
    x = dev(B.x)
    ho, wo = (B.h - 1) // B.stride + 1, (B.w - 1) // B.stride + 1
    need = P.prom_block_workspace_size(B.n, B.h, B.w, B.cin, B.chid, B.cout, B.stride)
    assert need <= P.prom_block_noalloc_max_workspace()
    ws = torch.empty(need, dtype=torch.int8, device=x.device)
    y_ref = torch.full((B.n, ho, wo, B.cout), 0x55, dtype=torch.int8, device=x.device)
    y_new = torch.full((B.n, ho, wo, B.cout), 0x2A, dtype=torch.int8, device=x.device)
    P.prom_block(x, B.chid, B.cout, B.stride, we, rqs[0], wd, rqs[1], wp, rqs[2], B.add_residual, ws, y=y_ref)
    P.prom_block_noalloc(x, B.chid, B.cout, B.stride, we, rqs[0], wd, rqs[1], wp, rqs[2], B.add_residual, y_new)
    torch.cuda.synchronize()
    want, _, _ = oracle.block(B.x, (e.weight, e.bias, e.mult, e.shift, e.act_min, e.act_max),
                              (d.weight, d.bias, d.mult, d.shift, d.act_min, d.act_max),
                              (p.weight, p.bias, p.mult, p.shift, p.act_min, p.act_max), B.stride, B.add_residual)
    return y_new.cpu().numpy(), y_ref.cpu().numpy(), want


def test_noalloc_block_two_calls_second_smaller(P):
    """Both shapes take the three-launch form (the one whose kernels use the scratch array; their
    hidden widths, 360 and 72 channels, are not a multiple of 16, which the one-kernel forms
    need): the second is smaller in every dimension, so it finds the first call's bytes in the
    array."""
    shapes = [(7001, 3, 14, 14, 60, 6, 60, 1), (7002, 2, 9, 7, 12, 6, 24, 2)]
    for seed, n, h, w, cin, t, cout, stride in shapes:
        B = make_block(seed, n, h, w, cin, t, cout, stride, signed_x=True)
        assert not P.prom_block_is_fused(n, h, w, cin, cin * t, cout, stride)
        got, ref, want = _run_both(P, B)
        assert_same(got, ref, f"prom_block_noalloc vs prom_block {(n, h, w, cin, t, cout, stride)}")
        assert_same(got, want, f"prom_block_noalloc vs oracle {(n, h, w, cin, t, cout, stride)}")


def test_noalloc_block_fused_form_and_limit(P):
    """A shape the library runs as one fused kernel goes through the same entry point; a shape
    whose intermediates exceed the fixed array is refused before anything is enqueued."""
    torch = torch_cuda()
    B = make_block(7003, 28, 28, 28, 32, 6)
    assert P.prom_block_is_fused(B.n, B.h, B.w, B.cin, B.chid, B.cout, 1)
    got, ref, want = _run_both(P, B)
    assert_same(got, ref, "prom_block_noalloc vs prom_block (fused form)")
    assert_same(got, want, "prom_block_noalloc vs oracle (fused form)")
    # 64 x 56 x 56 x 144 x 2 intermediates = 57.8 MB > 32 MiB
    big = make_block(7004, 1, 4, 4, 24, 6)
    e, d, p = big.expand, big.dw, big.project
    rqs = [requant_dev(P, l) for l in (e, d, p)]
    x = torch.zeros((64, 56, 56, 24), dtype=torch.int8, device="cuda")
    y = torch.full((64, 56, 56, 24), 7, dtype=torch.int8, device="cuda")
    assert P.prom_block_workspace_size(64, 56, 56, 24, 144, 24, 1) > P.prom_block_noalloc_max_workspace()
    with pytest.raises(P.PromError) as err:
        P.prom_block_noalloc(x, 144, 24, 1, dev(P.prom_pack_ternary(e.weight)), rqs[0], dev(d.weight), rqs[1],
                             dev(P.prom_pack_ternary(p.weight)), rqs[2], True, y)
    assert err.value.code == -7
    torch.cuda.synchronize()
    assert int((y != 7).sum()) == 0
