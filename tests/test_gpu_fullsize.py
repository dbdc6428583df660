"""Parity at the full benchmark sizes: every pointwise layer of the MobileNetV2 batch-128
sweep, launched exactly as bench.py launches it (prom_pw_conv_sequence, library plan), with
EVERY output element compared with the CPU oracle, on several runs in a row (a wrong value that
shows only now and then, such as a register reused too early after a store, has to show here).
The residual projection layers are checked on sampled pixel rows (a pointwise output row
depends only on its own input row, so the oracle can compute any row by itself)."""
import numpy as np
import pytest

import oracle
from workloads import make_pw_layer, mobilenetv2_pointwise_layers
from gpu_util import torch_cuda, dev, requant_dev

pytestmark = pytest.mark.gpu
BATCH = 128
SEED = 0x50524F4D + 300  # the seeds bench.py uses


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def _sample_rows(m, rng):
    fixed = np.concatenate([np.arange(0, min(m, 200)), np.arange(max(0, m - 200), m),
                            np.arange(max(0, m // 2 - 64), min(m, m // 2 + 64))])
    rnd = rng.integers(0, m, size=1500)
    return np.unique(np.concatenate([fixed, rnd]))


def test_mobilenetv2_sweep_batch128_every_output(P):
    torch = torch_cuda()
    shapes = mobilenetv2_pointwise_layers()
    layers, wants = [], []
    for i, s in enumerate(shapes):
        L = make_pw_layer(SEED + i, BATCH, s.hw, s.hw, s.cin, s.cout)
        x = dev(L.x)
        y = torch.full((BATCH, s.hw, s.hw, s.cout), -77, dtype=torch.int8, device="cuda")
        layers.append((x, dev(P.prom_pack_ternary(L.weight)), s.cout, requant_dev(P, L), None, y))
        wants.append(dev(oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, L.act_min, L.act_max)))
    seq = P.PwSequence(layers)
    for run in range(4):
        for (_, _, _, _, _, y) in layers:
            y.fill_(-77)
        seq.run()
        torch.cuda.synchronize()
        for s, want, (_, _, _, _, _, y) in zip(shapes, wants, layers):
            bad = int((y != want).sum())
            assert bad == 0, f"run {run}, {s.name}: {bad} of {y.numel()} outputs differ from the oracle"


def test_projection_layers_with_residual_batch128(P):
    """The ten stride-1 projection layers with their skip connection (clamp to [-128,127], then
    saturating add), full size, sampled rows."""
    torch = torch_cuda()
    rng = np.random.default_rng(8)
    for i, s in enumerate(mobilenetv2_pointwise_layers()):
        if not s.residual:
            continue
        L = make_pw_layer(SEED + 500 + i, BATCH, s.hw, s.hw, s.cin, s.cout, act_window=(-128, 127),
                          with_residual=True)
        y = P.prom_pw_conv(dev(L.x), dev(P.prom_pack_ternary(L.weight)), s.cout, requant_dev(P, L),
                           dev(L.residual))
        torch.cuda.synchronize()
        m = BATCH * s.hw * s.hw
        rows = _sample_rows(m, rng)
        xs = L.x.reshape(m, s.cin)[rows].reshape(1, 1, len(rows), s.cin)
        rs = L.residual.reshape(m, s.cout)[rows].reshape(1, 1, len(rows), s.cout)
        want = oracle.pw_conv(xs, L.weight, L.bias, L.mult, L.shift, -128, 127, rs).reshape(len(rows), s.cout)
        got = y.view(m, s.cout)[torch.from_numpy(rows).cuda()].cpu().numpy()
        assert np.array_equal(got, want), f"{s.name}: sampled outputs differ"
