"""Pins of the weight-quantiser oracle against things other than itself: worked examples done by
hand, the closed-form ternary distribution the paper derives for Kaiming-initialised weights
(its appendix on the weight distribution at initialisation: about 31 % zeros, 34.5 % each of
+1 and -1), invariances, and the paper's own pseudocode run with PyTorch CPU ops."""
import numpy as np
import pytest

import oracle


def test_absmean_hand_example_and_ties():
    # row 0: mean |w| = 0.15 -> w/mean = 0.667, -1.333, 2, 0 -> 1, -1, clamp(2) = 1, 0
    # row 1: mean = 1: 0.5 -> 0 and -0.5 -> 0 (half to even), 1.5 -> 2 -> 1, -1.5 -> -2 -> -1,
    #        chosen so that the mean is exactly 1: |0.5|+|0.5|+|1.5|+|1.5| = 4
    w = np.array([[0.1, -0.2, 0.3, 0.0], [0.5, -0.5, 1.5, -1.5]], dtype=np.float32)
    q, scale = oracle.quantize_pw_absmean(w)
    assert q.tolist() == [[1, -1, 1, 0], [0, 0, 1, -1]]
    assert scale[1] == np.float32(1.0)
    assert abs(scale[0] - 1 / 0.15) < 1e-5


def test_absmean_zero_row_and_eps():
    w = np.zeros((2, 8), dtype=np.float32)
    w[1, 3] = 4e-5  # mean 5e-6 < eps: the scale is 1/eps, 4e-5 * 1e5 = 4 -> clamp 1
    q, scale = oracle.quantize_pw_absmean(w, eps=1e-5)
    assert not q[0].any() and np.allclose(scale, 1e5, rtol=1e-6)
    assert q[1].tolist() == [0, 0, 0, 1, 0, 0, 0, 0]


def test_absmean_closed_form_distribution_at_initialisation():
    # Kaiming normal weights, sigma = sqrt(2/cout): w/alpha is N(0, pi/2) and the share between the
    # rounding thresholds -1/2 and 1/2 is erf(0.5 / sqrt(pi)) = 0.3101; the rest splits evenly
    from math import erf, pi, sqrt
    rng = np.random.default_rng(1)
    cout, cin = 384, 4096
    w = (rng.standard_normal((cout, cin)) * sqrt(2.0 / cout)).astype(np.float32)
    q, _ = oracle.quantize_pw_absmean(w)
    p0 = float((q == 0).mean())
    assert abs(erf(0.5 / sqrt(pi)) - 0.3101) < 1e-3
    assert abs(p0 - 0.3101) < 0.003            # the paper: "approximately 31 %"
    assert abs(float((q == 1).mean()) - 0.345) < 0.003 and abs(float((q == -1).mean()) - 0.345) < 0.003


def test_absmean_is_scale_invariant_and_odd():
    rng = np.random.default_rng(2)
    w = rng.standard_normal((16, 100)).astype(np.float32)
    q, s = oracle.quantize_pw_absmean(w)
    q8, s8 = oracle.quantize_pw_absmean(w * np.float32(8.0))   # a power of two: exact in float32
    assert np.array_equal(q, q8) and np.array_equal(s, s8 * np.float32(8.0))
    qn, _ = oracle.quantize_pw_absmean(-w)
    assert np.array_equal(qn, -q)


def test_absmax_hand_example():
    w = np.zeros((2, 3, 3), dtype=np.float32)
    w[0] = np.array([[1.0, -2.0, 0.5], [0.0, 0.25, -0.004], [2.0, 1.99, -1.0]])
    w[1, 1, 1] = -3.0
    q, scale = oracle.quantize_dw_absmax(w)
    assert q.shape == (3, 3, 2) and scale[0] == np.float32(63.5) and abs(scale[1] - 127 / 3) < 1e-5
    # 63.5 * (1, -2, .5, 0, .25, -.004, 2, 1.99, -1) = 63.5, -127, 31.75, 0, 15.875, -0.254, 127, 126.365, -63.5
    # half to even: 63.5 -> 64, -63.5 -> -64
    assert q[:, :, 0].tolist() == [[64, -127, 32], [0, 16, 0], [127, 126, -64]]
    assert q[1, 1, 1] == -127 and np.count_nonzero(q[:, :, 1]) == 1


def test_absmax_extremes_map_to_127_and_layout():
    rng = np.random.default_rng(3)
    w = rng.standard_normal((40, 3, 3)).astype(np.float32)
    q, _ = oracle.quantize_dw_absmax(w)
    for c in range(40):
        k = np.unravel_index(np.argmax(np.abs(w[c])), (3, 3))
        assert abs(int(q[k[0], k[1], c])) == 127 and np.sign(q[k[0], k[1], c]) == np.sign(w[c][k])
    assert np.abs(q.astype(int)).max() == 127  # -128 is never produced by a symmetric absmax scale


def test_against_the_papers_pseudocode_in_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(4)
    w = rng.standard_normal((96, 160)).astype(np.float32)
    t = torch.from_numpy(w)
    scale = 1.0 / t.abs().mean(dim=-1, keepdim=True).clamp_(min=1e-5)
    want = (t * scale).round().clamp_(-1, 1).numpy().astype(np.int8)
    q, s = oracle.quantize_pw_absmean(w)
    # torch's float32 mean may differ from the float64-summed one in the last bit; a code can then
    # differ only where w*scale sits within that bit of a rounding threshold
    assert (q != want).mean() < 1e-4
    assert np.allclose(s, scale.numpy().ravel(), rtol=3e-7)
    d = rng.standard_normal((64, 3, 3)).astype(np.float32)
    td = torch.from_numpy(d)
    sd = 127.0 / td.abs().flatten(start_dim=1).max(dim=-1, keepdim=True).values.clamp_(min=1e-5)
    wantd = (td.flatten(start_dim=1) * sd).round().clamp_(-128, 127).numpy().astype(np.int8).reshape(64, 3, 3)
    qd, s2 = oracle.quantize_dw_absmax(d)
    # torch evaluates 127.0 / t as reciprocal(t) * 127, one rounding more than the single division
    # taken here: scales agree to the last bit or so, codes wherever w*scale is not on a threshold
    assert (qd != np.transpose(wantd, (1, 2, 0))).mean() < 1e-3 and np.allclose(s2, sd.numpy().ravel(), rtol=3e-7)


def test_activation_absmax_hand_example_and_properties():
    x = np.zeros((3, 2, 2, 2), dtype=np.float32)
    x[0].reshape(-1)[:] = [2.0, -1.0, 0.5, 0.0, 0.0078125, 1.0, -2.0, 0.25]   # absmax 2 -> scale 63.5
    x[2].reshape(-1)[:] = [1e-7, 0, 0, 0, 0, 0, 0, -2e-7]                      # below eps: scale 127/eps
    q, scale = oracle.quantize_activation_absmax(x, eps=1e-5)
    # 63.5 * (2, -1, .5, 0, 2^-7, 1, -2, .25) = 127, -63.5 -> -64 (even), 31.75 -> 32, 0, 0.496 -> 0, 63.5 -> 64, -127, 15.875 -> 16
    assert q[0].reshape(-1).tolist() == [127, -64, 32, 0, 0, 64, -127, 16]
    assert scale[0] == np.float32(63.5)
    assert not q[1].any() and scale[1] == np.float32(127.0) / np.float32(1e-5)
    # 1e-7 * 1.27e7 = 1.27 -> 1, -2e-7 -> -2.54 -> -3
    assert q[2].reshape(-1).tolist() == [1, 0, 0, 0, 0, 0, 0, -3]
    rng = np.random.default_rng(5)
    y = rng.standard_normal((4, 7, 5, 3)).astype(np.float32) * np.float32(3.0)
    qy, sy = oracle.quantize_activation_absmax(y)
    for i in range(4):                      # the extreme element of every image maps to +-127
        k = np.argmax(np.abs(y[i]))
        assert abs(int(qy[i].reshape(-1)[k])) == 127
    q2, s2 = oracle.quantize_activation_absmax(y * np.float32(4.0))   # power of two: same codes
    assert np.array_equal(q2, qy) and np.array_equal(s2 * np.float32(4.0), sy)
    # images are independent: quantising one alone gives the same codes
    q1, _ = oracle.quantize_activation_absmax(y[2:3])
    assert np.array_equal(q1[0], qy[2])


def test_activation_absmax_against_the_papers_pseudocode_in_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(6)
    x = rng.standard_normal((5, 16, 9, 9)).astype(np.float32)
    t = torch.from_numpy(x)
    scale = 127.0 / t.abs().flatten(start_dim=1).max(dim=-1, keepdim=True).values.clamp_(min=1e-5)
    want = (t.flatten(start_dim=1) * scale).round().clamp_(-128, 127).numpy().astype(np.int8).reshape(x.shape)
    q, s = oracle.quantize_activation_absmax(x)
    assert (q != want).mean() < 1e-3 and np.allclose(s, scale.numpy().ravel(), rtol=3e-7)


def test_gconv_absmax_pins():
    """Grouped 3x3 weights: one absmax scale per output channel over its group's input channels
    and the 9 taps (Section 3.1: W[c_out][c_in][K][K], Eq. 4-5).  Group size 1 is the (pinned)
    depthwise quantiser; the extreme of every channel maps to +-127; each code is within half a
    step of w * scale; torch's statement of the pseudocode agrees up to its extra rounding."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(6)
    d = rng.standard_normal((24, 1, 3, 3)).astype(np.float32)
    q1, s1 = oracle.quantize_gconv_absmax(d)
    q0, s0 = oracle.quantize_dw_absmax(d.reshape(24, 3, 3))
    assert np.array_equal(q1.reshape(3, 3, 24), q0) and np.array_equal(s1, s0)
    w = (rng.standard_normal((32, 8, 3, 3)) * rng.uniform(0.01, 3.0, (32, 1, 1, 1))).astype(np.float32)
    q, s = oracle.quantize_gconv_absmax(w)
    assert q.shape == (3, 3, 32, 8) and s.shape == (32,)
    for c in range(32):
        k = np.unravel_index(np.argmax(np.abs(w[c])), (8, 3, 3))
        assert abs(int(q[k[1], k[2], c, k[0]])) == 127 and np.sign(q[k[1], k[2], c, k[0]]) == np.sign(w[c][k])
        assert s[c] == np.float32(127.0) / np.abs(w[c]).max()
    back = np.transpose(q, (2, 3, 0, 1)).astype(np.float64)          # [c][gs][3][3]
    assert np.all(np.abs(back - w.astype(np.float64) * s[:, None, None, None].astype(np.float64)) <= 0.5 + 1e-4)
    t = torch.from_numpy(w)
    st = 127.0 / t.abs().flatten(start_dim=1).max(dim=-1, keepdim=True).values.clamp_(min=1e-5)
    want = (t.flatten(start_dim=1) * st).round().clamp_(-128, 127).numpy().astype(np.int8).reshape(32, 8, 3, 3)
    assert (np.transpose(q, (2, 3, 0, 1)) != want).mean() < 1e-3
    z, sz = oracle.quantize_gconv_absmax(np.zeros((4, 4, 3, 3), np.float32))
    assert not z.any() and np.all(sz == np.float32(127.0) / np.float32(1e-5))
