"""Parity on the pointwise layers of the two other architecture families of the paper's
evaluation (Section 5: RegNetX and ResNeXt): RegNetX-400MF (32..384 channels, all bandwidth- or
latency-bound) and ResNeXt-50 32x4d (64..2048 channels; the layers of its last two stages have
more operations per byte than the matrix units' balance point).  Every unique shape with every
output element at a small batch, and all of them in one prom_pw_conv_sequence call at the
benchmark's batch on sampled pixel rows (a pointwise output row depends only on its input row)."""
import numpy as np
import pytest

import oracle
from workloads import make_pw_layer, regnetx_400mf_pointwise_layers, resnext50_32x4d_pointwise_layers
from gpu_util import torch_cuda, dev, requant_dev, assert_same

pytestmark = pytest.mark.gpu
FAMILIES = {"regnetx_400mf": (regnetx_400mf_pointwise_layers, 4),
            "resnext50_32x4d": (resnext50_32x4d_pointwise_layers, 2)}


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    P.load_library()
    return P


def unique_shapes(layers):
    seen, out = set(), []
    for s in layers:
        key = (s.hw, s.cin, s.cout, s.residual)
        if key not in seen:
            seen.add(key)
            out.append(s)
    return out


@pytest.mark.parametrize("family", sorted(FAMILIES))
def test_every_unique_shape_every_output(P, family):
    torch = torch_cuda()
    layers_of, batch = FAMILIES[family]
    for i, s in enumerate(unique_shapes(layers_of())):
        window = (-128, 127) if s.residual else (0, 127)
        L = make_pw_layer(9100 + i, batch, s.hw, s.hw, s.cin, s.cout, act_window=window,
                          with_residual=s.residual)
        y = P.prom_pw_conv(dev(L.x), dev(P.prom_pack_ternary(L.weight)), s.cout, requant_dev(P, L),
                           dev(L.residual) if s.residual else None)
        torch.cuda.synchronize()
        want = oracle.pw_conv(L.x, L.weight, L.bias, L.mult, L.shift, L.act_min, L.act_max, L.residual)
        assert_same(y.cpu().numpy(), want, f"{family} {s.name} ({s.hw}x{s.hw}, {s.cin}->{s.cout})")


def _sample_rows(m, rng):
    fixed = np.concatenate([np.arange(0, min(m, 160)), np.arange(max(0, m - 160), m)])
    return np.unique(np.concatenate([fixed, rng.integers(0, m, size=700)]))


@pytest.mark.parametrize("batch", [128, 32])
@pytest.mark.parametrize("family", sorted(FAMILIES))
def test_sequence_at_batch128_sampled_rows(P, family, batch):
    """The configuration the benchmark leg times: all unique shapes at batch 128 through one
    prom_pw_conv_sequence call (independent layers: the library may share launches).  Also at
    batch 32, where the shared launches take smaller pieces and layers with a thousand and more
    input channels leave the kernel for wide layers and may share a launch."""
    torch = torch_cuda()
    rng = np.random.default_rng(12)
    shapes = unique_shapes(FAMILIES[family][0]())
    inputs, layers = [], []
    for i, s in enumerate(shapes):
        window = (-128, 127) if s.residual else (0, 127)
        L = make_pw_layer(9300 + i, batch, s.hw, s.hw, s.cin, s.cout, act_window=window,
                          with_residual=s.residual)
        y = torch.full((batch, s.hw, s.hw, s.cout), -77, dtype=torch.int8, device="cuda")
        layers.append((dev(L.x), dev(P.prom_pack_ternary(L.weight)), s.cout, requant_dev(P, L),
                       dev(L.residual) if s.residual else None, y))
        inputs.append(L)
    seq = P.PwSequence(layers)
    for run in range(2):
        seq.run()
        torch.cuda.synchronize()
        for s, L, lay in zip(shapes, inputs, layers):
            m = batch * s.hw * s.hw
            rows = _sample_rows(m, rng)
            xs = L.x.reshape(m, s.cin)[rows].reshape(1, 1, len(rows), s.cin)
            rs = L.residual.reshape(m, s.cout)[rows].reshape(1, 1, len(rows), s.cout) if s.residual else None
            want = oracle.pw_conv(xs, L.weight, L.bias, L.mult, L.shift, L.act_min, L.act_max, rs)
            got = lay[5].view(m, s.cout)[torch.from_numpy(rows).cuda()].cpu().numpy()
            assert_same(got, want.reshape(len(rows), s.cout), f"run {run}, {family} {s.name}")
            lay[5].fill_(-77)
