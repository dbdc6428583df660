"""Pins of the oracle of the pointwise layer with the paper's dynamic per-image activation scale
(Section 3.1, Eq. 6-7 applied to the layer's real-valued output) against things other than
itself: a worked example done by hand, the composition of the two oracles that already exist and
are pinned on their own (integer accumulators from the C oracle, then the activation quantiser),
and invariances that a wrong image index, a dropped bias or a transposed operand would break."""
import numpy as np

import oracle
from workloads import make_pw_layer


def test_hand_example():
    # one image, two pixels, cin 4, cout 2; w_scale (0.5, 0.25), x_step 0.5, bias (1, -2)
    # pixel 0: x = (8, -4, 2, 0):  acc0 = 8+4+0+0 = 12 (w0 = +,-,0,+), acc1 = -8-4+2 = -10 (w1 = -,+,+,0)
    #          z = 12*.5*.5 + 1 = 4;  -10*.25*.5 - 2 = -3.25
    # pixel 1: x = (0, 16, -16, 4): acc0 = 0-16+0+4 = -12, acc1 = 0+16-16 = 0
    #          z = -12*.25 + 1 = -2;  0 - 2 = -2
    # amax = 4, scale = 31.75: q = 127, -103.1875 -> -103, -63.5 -> -64 (half to even), -64
    x = np.array([[[[8, -4, 2, 0], [0, 16, -16, 4]]]], dtype=np.int8)
    wt = np.array([[1, -1, 0, 1], [-1, 1, 1, 0]], dtype=np.int8)
    q, amax, scale = oracle.pw_conv_dynamic_quant(x, wt, [0.5], [0.5, 0.25], [1.0, -2.0])
    assert amax.tolist() == [4.0] and scale.tolist() == [31.75]
    assert q.reshape(2, 2).tolist() == [[127, -103], [-64, -64]]
    # with ReLU the negative values go to 0 and the scale is unchanged
    q, amax, scale = oracle.pw_conv_dynamic_quant(x, wt, [0.5], [0.5, 0.25], [1.0, -2.0], relu=True)
    assert q.reshape(2, 2).tolist() == [[127, 0], [0, 0]] and amax.tolist() == [4.0]
    # without the bias: z = 3, -1.25, -3, 0 -> amax 3, scale 42.333332: 127, -52.9 -> -53, -127, 0
    q, amax, _ = oracle.pw_conv_dynamic_quant(x, wt, [0.5], [0.5, 0.25])
    assert q.reshape(2, 2).tolist() == [[127, -53], [-127, 0]] and amax.tolist() == [3.0]


def _random_case(seed, n, hw, cin, cout):
    L = make_pw_layer(seed, n, hw, hw, cin, cout, signed_x=True)
    rng = np.random.default_rng(seed)
    x_step = (rng.uniform(0.002, 0.05, n) * 2.0 ** rng.integers(-3, 4, n)).astype(np.float32)
    w_scale = rng.uniform(0.01, 0.2, cout).astype(np.float32)
    bias = rng.normal(0, 0.5, cout).astype(np.float32)
    return L, x_step, w_scale, bias


def test_equals_the_composition_of_the_two_pinned_oracles():
    for seed, (n, hw, cin, cout), relu in ((1, (3, 5, 24, 40), False), (2, (2, 7, 100, 16), True),
                                           (3, (4, 3, 8, 8), False)):
        L, x_step, w_scale, bias = _random_case(seed, n, hw, cin, cout)
        q, amax, scale = oracle.pw_conv_dynamic_quant(L.x, L.weight, x_step, w_scale, bias, relu)
        acc = oracle.pw_accum(L.x, L.weight)                     # the C oracle's integer accumulators
        z = np.empty(acc.shape, dtype=np.float32)
        for i in range(n):                                       # the dequantisation, image by image
            t = acc[i].astype(np.float32) * w_scale
            z[i] = t * x_step[i] + bias
        if relu:
            z[z < 0] = 0
        q2, scale2 = oracle.quantize_activation_absmax(z)
        assert np.array_equal(q, q2) and np.array_equal(scale, scale2)
        assert np.array_equal(amax, np.abs(z).reshape(n, -1).max(axis=1))


def test_invariances():
    L, x_step, w_scale, bias = _random_case(7, 3, 6, 32, 24)
    q, amax, scale = oracle.pw_conv_dynamic_quant(L.x, L.weight, x_step, w_scale, None)
    # every image uses its whole range: its largest value maps to +-127
    assert (np.abs(q.astype(np.int32)).reshape(3, -1).max(axis=1) == 127).all()
    # a power-of-two change of one image's input step scales that image's amax and nothing else
    xs2 = x_step.copy()
    xs2[1] *= np.float32(4.0)
    q2, amax2, _ = oracle.pw_conv_dynamic_quant(L.x, L.weight, xs2, w_scale, None)
    assert np.array_equal(q2, q) and amax2[1] == amax[1] * 4 and amax2[0] == amax[0] and amax2[2] == amax[2]
    # images are independent: image 2 alone gives the same codes
    q1, a1, _ = oracle.pw_conv_dynamic_quant(L.x[2:3], L.weight, x_step[2:3], w_scale, None)
    assert np.array_equal(q1[0], q[2]) and a1[0] == amax[2]
    # permuting the pixels of an image permutes its codes; permuting output channels too
    perm = np.random.default_rng(3).permutation(36)
    xp = L.x.reshape(3, 36, 32)[:, perm].reshape(3, 6, 6, 32)
    qp, _, _ = oracle.pw_conv_dynamic_quant(xp, L.weight, x_step, w_scale, None)
    assert np.array_equal(qp.reshape(3, 36, 24), q.reshape(3, 36, 24)[:, perm])
    cperm = np.random.default_rng(4).permutation(24)
    qc, _, _ = oracle.pw_conv_dynamic_quant(L.x, L.weight[cperm], x_step, w_scale[cperm], None)
    assert np.array_equal(qc, q[..., cperm])
    # negating the weights negates the codes (no bias, no ReLU; -128 cannot occur: |z| <= amax)
    qn, _, _ = oracle.pw_conv_dynamic_quant(L.x, -L.weight, x_step, w_scale, None)
    assert np.array_equal(qn, -q)
    # ReLU: no negative code, and the positive codes are those of the plain form whenever the
    # image's maximum is a positive value
    qr, ar, _ = oracle.pw_conv_dynamic_quant(L.x, L.weight, x_step, w_scale, None, relu=True)
    assert qr.min() >= 0
    for i in range(3):
        if ar[i] == amax[i]:
            assert np.array_equal(qr[i], np.maximum(q[i], 0))


def test_zero_image_and_eps():
    x = np.zeros((2, 2, 2, 8), dtype=np.int8)
    x[1, 0, 0, 0] = 1
    wt = np.ones((4, 8), dtype=np.int8)
    q, amax, scale = oracle.pw_conv_dynamic_quant(x, wt, [1.0, 1e-6], [1.0] * 4, None, eps=1e-5)
    assert amax[0] == 0 and scale[0] == np.float32(127.0) / np.float32(1e-5) and not q[0].any()
    # image 1: z = 1e-6 < eps: scale 127/eps, code round(1e-6 * 1.27e7) = 13
    assert amax[1] == np.float32(1e-6) and q[1, 0, 0].tolist() == [13] * 4 and not q[1, 1].any()
