"""The pointwise layer tables of the two other families of the paper's evaluation (Section 5),
against what their public architecture tables fix: block counts, channel ranges, resolutions and
the chaining of consecutive blocks."""
from workloads import regnetx_400mf_pointwise_layers, resnext50_32x4d_pointwise_layers


def test_layer_tables():
    r, x = regnetx_400mf_pointwise_layers(), resnext50_32x4d_pointwise_layers()
    assert len(r) == 2 * 22 + 4 and len(x) == 2 * 16 + 4   # two 1x1 per block, one shortcut per stage
    assert max(s.cout for s in r) == 384 and max(s.cout for s in x) == 2048
    assert (r[0].hw, r[0].cin, r[-1].hw) == (112, 32, 7) and (x[0].hw, x[0].cin, x[-1].hw) == (56, 64, 7)
    # a block's last 1x1 feeds the next block's first
    for fam in (r, x):
        prev = None
        for s in fam:
            if s.name.endswith(".reduce") and prev is not None:
                assert s.cin == prev.cout and s.hw == prev.hw
            if s.name.endswith(".expand"):
                prev = s
