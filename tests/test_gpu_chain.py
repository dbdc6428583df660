"""The whole MobileNetV2 body as a chain: the 17 inverted-residual blocks in network order (the
four stride-2 depthwise layers included), each block fed with the previous block's output, then
the 1x1 head.  Block 1 has no expansion convolution (depthwise + projection calls); blocks 2-17
go through prom_block, which fuses the shapes it can and runs the others as three launches.
Every block output is compared with the oracle's, which walks the same chain on the CPU, for
ternary weights with the zero fractions the paper reports at initialisation and after training
(appendix A on the distribution of ternary weights: about 0.31 at initialisation, up to 0.55
in one layer after training; 0.5 in between)."""
import numpy as np
import pytest

import oracle
from workloads import SplitMix64, make_block, make_dw_layer, make_pw_layer, mobilenetv2_blocks
from gpu_util import assert_same, dev, requant_dev, torch_cuda

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def _pw_shift(k):
    """A shift range that keeps the output of a k-input ternary layer spread over the int8 range
    (accumulator spread grows with sqrt(k)); with the generators' default range a chain of layers
    collapses to per-channel constants after two layers."""
    s = max(0, int(round(np.log2(np.sqrt(k) + 1.0))))
    return (s, s + 1)


DW_SHIFT = (8, 9)


def _tup(l):
    return (l.weight, l.bias, l.mult, l.shift, l.act_min, l.act_max)


@pytest.mark.parametrize("p_zero,input_hw,n", [(0.5, 32, 2), (0.31, 16, 3), (0.55, 20, 1)])
def test_mobilenetv2_block_chain(P, p_zero, input_hw, n):
    torch = torch_cuda()
    blocks = mobilenetv2_blocks(input_hw)
    seed = 7700 + int(p_zero * 100)
    x_host = SplitMix64(seed).bytes_masked(n * input_hw * input_hw * blocks[0].cin, 0x7F).view(np.int8)
    x_host = x_host.reshape(n, input_hw, input_hw, blocks[0].cin)
    x_dev = dev(x_host)
    fused = []
    for i, b in enumerate(blocks):
        hw = b.hw_in
        if b.t == 1:
            D = make_dw_layer(seed + 10 * i + 1, n, hw, hw, b.cin, b.stride, act_window=(0, 127),
                              shift_range=DW_SHIFT, make_x=False)
            Q = make_pw_layer(seed + 10 * i + 2, n, hw, hw, b.cin, b.cout, act_window=(-128, 127),
                              p_zero=p_zero, shift_range=_pw_shift(b.cin), make_x=False)
            t = P.prom_dw_conv(x_dev, dev(D.weight), b.stride, requant_dev(P, D))
            y_dev = P.prom_pw_conv(t, dev(P.prom_pack_ternary(Q.weight)), b.cout, requant_dev(P, Q))
            th = oracle.dw_conv(x_host, D.weight, b.stride, D.bias, D.mult, D.shift, 0, 127)
            y_host = oracle.pw_conv(th, Q.weight, Q.bias, Q.mult, Q.shift, -128, 127)
        else:
            B = make_block(seed + 10 * i, n, hw, hw, b.cin, b.t, b.cout, b.stride, p_zero=p_zero,
                           expand_shift=_pw_shift(b.cin), dw_shift=DW_SHIFT,
                           project_shift=_pw_shift(b.cin * b.t))
            ws = torch.empty(P.prom_block_workspace_size(n, hw, hw, b.cin, B.chid, b.cout, b.stride),
                             dtype=torch.int8, device="cuda")
            # the fused kernel wherever it applies (at these small sizes the library itself would
            # take the three launches), the three launches elsewhere
            can = P.prom_block_can_fuse(n, hw, hw, b.cin, B.chid, b.cout, b.stride)
            y_dev = P.prom_block(x_dev, B.chid, b.cout, b.stride,
                                 dev(P.prom_pack_ternary(B.expand.weight)), requant_dev(P, B.expand),
                                 dev(B.dw.weight), requant_dev(P, B.dw),
                                 dev(P.prom_pack_ternary(B.project.weight)), requant_dev(P, B.project),
                                 B.add_residual, ws, path=P.BLOCK_FUSED if can else P.BLOCK_AUTO)
            y_host, _, _ = oracle.block(x_host, _tup(B.expand), _tup(B.dw), _tup(B.project), b.stride,
                                        B.add_residual)
            fused.append(can)
        torch.cuda.synchronize()
        assert_same(y_dev.cpu().numpy(), y_host, f"chain p_zero={p_zero} {b.name}")
        assert len(np.unique(y_host)) > 24, f"{b.name}: the chain's activations degenerated"
        x_dev, x_host = y_dev, y_host
    # the chain must exercise both forms of prom_block
    assert any(fused) and not all(fused)
    hw = x_host.shape[1]
    H = make_pw_layer(seed + 999, n, hw, hw, blocks[-1].cout, 1280, p_zero=p_zero,
                      shift_range=_pw_shift(blocks[-1].cout), make_x=False)
    y_dev = P.prom_pw_conv(x_dev, dev(P.prom_pack_ternary(H.weight)), 1280, requant_dev(P, H))
    torch.cuda.synchronize()
    assert_same(y_dev.cpu().numpy(), oracle.pw_conv(x_host, H.weight, H.bias, H.mult, H.shift, 0, 127), "head")


@pytest.mark.parametrize("n", [32, 128])
def test_mobilenetv2_block_chain_full_size_auto(P, n):
    """The 16 expanding blocks at the network's own sizes (224x224 input) through prom_block with
    PROM_BLOCK_AUTO, at batches where the library picks different forms: at 32 images every block
    is one kernel; at 128 the three blocks on the large maps are three launches and the thirteen
    behind them one kernel each.  Every output of every block against the oracle."""
    torch = torch_cuda()
    blocks = [b for b in mobilenetv2_blocks() if b.t != 1]
    seed = 8800 + n
    b0 = blocks[0]
    x_host = SplitMix64(seed).bytes_masked(n * b0.hw_in * b0.hw_in * b0.cin, 0x7F).view(np.int8)
    x_host = x_host.reshape(n, b0.hw_in, b0.hw_in, b0.cin)
    x_dev = dev(x_host)
    one_kernel = []
    for i, b in enumerate(blocks):
        hw = b.hw_in
        B = make_block(seed + 10 * i, 1, hw, hw, b.cin, b.t, b.cout, b.stride, expand_shift=_pw_shift(b.cin),
                       dw_shift=DW_SHIFT, project_shift=_pw_shift(b.cin * b.t))
        ws = torch.empty(P.prom_block_workspace_size(n, hw, hw, b.cin, B.chid, b.cout, b.stride),
                         dtype=torch.int8, device="cuda")
        one_kernel.append(P.prom_block_is_fused(n, hw, hw, b.cin, B.chid, b.cout, b.stride))
        y_dev = P.prom_block(x_dev, B.chid, b.cout, b.stride,
                             dev(P.prom_pack_ternary(B.expand.weight)), requant_dev(P, B.expand),
                             dev(B.dw.weight), requant_dev(P, B.dw),
                             dev(P.prom_pack_ternary(B.project.weight)), requant_dev(P, B.project),
                             B.add_residual, ws)
        y_host, _, _ = oracle.block(x_host, _tup(B.expand), _tup(B.dw), _tup(B.project), b.stride, B.add_residual)
        torch.cuda.synchronize()
        assert_same(y_dev.cpu().numpy(), y_host, f"full-size chain batch {n} {b.name}")
        del ws
        x_dev, x_host = y_dev, y_host
    if n == 32:
        assert all(one_kernel)
    else:
        assert one_kernel == [False] * 3 + [True] * 13


def test_chain_replays_from_a_captured_graph(P):
    """The library's calls on a stream can be captured in a HIP graph (no allocation, no memset,
    no host synchronisation inside a call once a shape has run): the 16 prom_block calls of the
    body are captured once and replayed with new inputs, with eager work and synchronisations
    between the replays; every replay must equal the eager result for the same input."""
    torch = torch_cuda()
    n, input_hw = 2, 32
    blocks = [b for b in mobilenetv2_blocks(input_hw) if b.t != 1]
    steps = []
    ws_bytes = 0
    x0 = torch.empty((n, blocks[0].hw_in, blocks[0].hw_in, blocks[0].cin), dtype=torch.int8, device="cuda")
    cur = x0
    for i, b in enumerate(blocks):
        hw, ho = b.hw_in, (b.hw_in - 1) // b.stride + 1
        B = make_block(7900 + i, 1, hw, hw, b.cin, b.t, b.cout, b.stride, expand_shift=_pw_shift(b.cin),
                       dw_shift=DW_SHIFT, project_shift=_pw_shift(b.cin * b.t))
        e, d, p = B.expand, B.dw, B.project
        y = torch.empty((n, ho, ho, b.cout), dtype=torch.int8, device="cuda")
        ws_bytes = max(ws_bytes, P.prom_block_workspace_size(n, hw, hw, b.cin, B.chid, b.cout, b.stride))
        path = P.BLOCK_FUSED if P.prom_block_can_fuse(n, hw, hw, b.cin, B.chid, b.cout, b.stride) else P.BLOCK_AUTO
        steps.append((cur, B.chid, b.cout, b.stride, dev(P.prom_pack_ternary(e.weight)), requant_dev(P, e),
                      dev(d.weight), requant_dev(P, d), dev(P.prom_pack_ternary(p.weight)), requant_dev(P, p),
                      B.add_residual, y, path))
        cur = y
    ws = torch.empty(ws_bytes, dtype=torch.int8, device="cuda")
    outs = [s[-2] for s in steps]

    def run_chain():
        for (xi, chid, cout, stride, we, rqe, wd, rqd, wp, rqp, addres, y, path) in steps:
            P.prom_block(xi, chid, cout, stride, we, rqe, wd, rqd, wp, rqp, addres, ws, y, path=path)

    def new_input(seed):
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)
        x0.copy_(torch.randint(0, 128, x0.shape, dtype=torch.int8, device="cuda", generator=g))

    new_input(1)
    run_chain()                       # warm-up: every shape has run once before the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run_chain()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for seed in (2, 3, 4):
        new_input(seed)
        run_chain()
        torch.cuda.synchronize()
        want = [o.clone() for o in outs]
        for o in outs:
            o.fill_(-77)              # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, (o, w) in enumerate(zip(outs, want)):
            assert torch.equal(o, w), f"replay for input {seed}: block {blocks[k].name} differs from the eager run"
