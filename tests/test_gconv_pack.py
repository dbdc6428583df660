"""Host logic of prom_gconv_pack (no GPU): the prepared form holds, per block of 64 channels and
kernel tap, the block-diagonal [64 x 64] weight matrix in the documented entry order."""
import numpy as np
import pytest

import paper_2505_03254_amd as P
from workloads import make_gconv_layer


@pytest.mark.parametrize("c,gs", [(16, 4), (64, 8), (96, 16), (160, 32), (128, 64), (40, 4)])
def test_fragments_hold_the_block_diagonal_matrices(c, gs):
    G = make_gconv_layer(800 + c + gs, 1, 3, 3, c, gs, make_x=False)
    frag = P.prom_gconv_pack(G.weight)
    ncb = (c + 63) // 64
    dense = np.zeros((9, ncb * 64, ncb * 64), dtype=np.int8)  # [tap][oc][ic]
    for oc in range(c):
        first = (oc // gs) * gs
        dense[:, oc, first:first + gs] = G.weight.reshape(9, c, gs)[:, oc, :]
    if gs <= 16:
        # taps in the k dimension: k group kg of step s is tap 4s + kg, taps 9..11 are zero
        assert frag.size == P.prom_gconv_frag_size(c, gs) == ncb * 4 * 3 * 64 * 16
        f = frag.view(np.int8).reshape(ncb, 4, 3, 64, 16)
        for cb in range(ncb):
            for t in range(4):
                for lane in range(64):
                    i, kg = lane & 15, lane >> 4
                    oc = 64 * cb + 16 * t + i
                    ic0 = 64 * cb + 16 * t
                    for s_ in range(3):
                        tap = 4 * s_ + kg
                        want = dense[tap, oc, ic0:ic0 + 16] if tap < 9 else np.zeros(16, np.int8)
                        assert np.array_equal(f[cb, t, s_, lane, :], want), (cb, t, s_, lane)
                    # nothing outside the tile's own 16 input channels is needed: the rest of the row is zero
                    row = dense[:, oc, :].copy()
                    row[:, ic0:ic0 + 16] = 0
                    assert not row.any()
        return
    assert frag.size == P.prom_gconv_frag_size(c, gs) == ncb * 4 * 9 * 64 * 16
    f = frag.view(np.int8).reshape(ncb, 4, 9, 64, 16)
    for cb in range(ncb):
        for t in range(4):
            for lane in range(64):
                i, kg = lane & 15, lane >> 4
                oc = 64 * cb + 16 * (i >> 2) + 4 * t + (i & 3)
                ic0 = 64 * cb + 16 * kg
                assert np.array_equal(f[cb, t, :, lane, :], dense[:, oc, ic0:ic0 + 16]), (cb, t, lane)


def test_sizes_and_errors():
    assert P.prom_gconv_frag_size(64, 5) == 0 and P.prom_gconv_frag_size(66, 4) == 0
    assert P.prom_gconv_frag_size(24, 16) == 0  # 24 % 16 != 0
    with pytest.raises(P.PromError) as e:
        P.prom_gconv_pack(np.zeros((3, 3, 10, 5), np.int8))
    assert e.value.code == -2
