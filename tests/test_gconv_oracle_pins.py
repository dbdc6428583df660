"""Pins of the oracle's grouped 3x3 convolution (RegNet / ResNeXt have group sizes above one
where MobileNetV2 has the depthwise conv: paper, Section 2; 8-bit weights with one scale per
output channel: Section 3.1, Eq. 4-5).

Pinned against: torch's conv2d with groups (a library routine, float64, exact for these
magnitudes), for several group sizes up to one dense group; the depthwise oracle at group size 1;
brute force in Python integers on tiny cases; group independence and a joint permutation of the
channels of a group; the requantisation, itself pinned, applied to the raw sums."""
import numpy as np
import pytest

import oracle
from workloads import make_gconv_layer, make_dw_layer, prelu_mult_neg


def _torch_grouped(x, weight, stride):
    torch = pytest.importorskip("torch")
    n, h, w, c = x.shape
    gs = weight.shape[3]
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    # torch layout [cout][cin per group][kh][kw]
    wt = torch.from_numpy(weight.astype(np.float64)).permute(2, 3, 0, 1).contiguous()
    out = torch.nn.functional.conv2d(xt, wt, stride=stride, padding=1, groups=c // gs)
    return np.rint(out.permute(0, 2, 3, 1).numpy()).astype(np.int64)


@pytest.mark.parametrize("c,gs", [(8, 1), (8, 2), (12, 4), (16, 8), (32, 16), (24, 24), (48, 24), (20, 5)])
@pytest.mark.parametrize("stride", [1, 2])
def test_raw_sums_match_library_grouped_conv(c, gs, stride):
    G = make_gconv_layer(700 + c + gs, 2, 7, 6, c, gs, stride, signed_x=True)
    acc = oracle.gconv3x3_accum(G.x, G.weight, stride)
    assert np.array_equal(acc.astype(np.int64), _torch_grouped(G.x, G.weight, stride))


def test_group_size_one_is_the_depthwise_oracle():
    for stride in (1, 2):
        D = make_dw_layer(710, 2, 6, 7, 12, stride, signed_x=True, act_window=(-128, 127))
        a = oracle.dw_conv(D.x, D.weight, stride, D.bias, D.mult, D.shift, -128, 127)
        b = oracle.gconv3x3(D.x, D.weight.reshape(3, 3, 12, 1), stride, D.bias, D.mult, D.shift, -128, 127)
        assert np.array_equal(a, b)


@pytest.mark.parametrize("h,w,stride", [(1, 1, 1), (2, 3, 1), (3, 2, 2), (4, 4, 2), (1, 5, 2)])
def test_brute_force_tiny(h, w, stride):
    c, gs = 6, 3
    G = make_gconv_layer(720 + h * 10 + w, 1, h, w, c, gs, stride, signed_x=True)
    acc = oracle.gconv3x3_accum(G.x, G.weight, stride)
    ho, wo = (h - 1) // stride + 1, (w - 1) // stride + 1
    for oy in range(ho):
        for ox in range(wo):
            for ch in range(c):
                tot = 0
                for i in range(3):
                    for j in range(3):
                        iy, ix = oy * stride + i - 1, ox * stride + j - 1
                        if 0 <= iy < h and 0 <= ix < w:
                            for k in range(gs):
                                tot += int(G.x[0, iy, ix, (ch // gs) * gs + k]) * int(G.weight[i, j, ch, k])
                assert int(acc[0, oy, ox, ch]) == tot


def test_groups_are_independent_and_channel_order_inside_a_group_is_a_convention():
    G = make_gconv_layer(730, 1, 5, 5, 12, 4, 1, signed_x=True)
    base = oracle.gconv3x3_accum(G.x, G.weight, 1)
    x2 = G.x.copy()
    x2[..., 4:8] = -x2[..., 4:8] // 2          # change group 1 only
    other = oracle.gconv3x3_accum(x2, G.weight, 1)
    assert np.array_equal(base[..., :4], other[..., :4]) and np.array_equal(base[..., 8:], other[..., 8:])
    assert not np.array_equal(base[..., 4:8], other[..., 4:8])
    # permute the input channels of group 2 and the matching weight columns: same sums
    perm = np.array([2, 0, 3, 1])
    x3 = G.x.copy()
    x3[..., 8:12] = G.x[..., 8 + perm]
    w3 = G.weight.copy()
    w3[:, :, 8:12, :] = G.weight[:, :, 8:12, :][..., perm]
    assert np.array_equal(base, oracle.gconv3x3_accum(x3, w3, 1))


def test_bytes_are_the_pinned_requantisation_of_the_raw_sums():
    G = make_gconv_layer(740, 2, 6, 5, 16, 8, 2, signed_x=True, shift_range=(9, 14))
    acc = oracle.gconv3x3_accum(G.x, G.weight, 2)
    y = oracle.gconv3x3(G.x, G.weight, 2, G.bias, G.mult, G.shift, -100, 90)
    mneg = prelu_mult_neg(740, G.mult)
    yp = oracle.gconv3x3(G.x, G.weight, 2, G.bias, G.mult, G.shift, -128, 127, mult_neg=mneg)
    it = np.nditer(acc, flags=["multi_index"])
    for a in it:
        ch = it.multi_index[3]
        s = int(a) + int(G.bias[ch])
        q = oracle.requant(s, int(G.mult[ch]), int(G.shift[ch]))
        assert int(y[it.multi_index]) == min(max(q, -100), 90)
        qp = oracle.requant_prelu(s, int(G.mult[ch]), int(mneg[ch]), int(G.shift[ch]))
        assert int(yp[it.multi_index]) == min(max(qp, -128), 127)


def test_rejects_bad_group_size():
    G = make_gconv_layer(750, 1, 3, 3, 8, 4)
    with pytest.raises(ValueError):
        oracle.gconv3x3_accum(G.x, np.zeros((3, 3, 8, 3), np.int8), 1)
