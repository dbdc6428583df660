"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares,
packs weights as documented and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def P():
    import paper_2505_03254_amd as P
    if not os.path.exists(P.library_path()):
        from paper_2505_03254_amd.build import build
        build()
    P.load_library()
    return P


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "prom.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(prom_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(P):
    lib = P.load_library()
    names = _declared_functions()
    assert {"prom_pw_conv", "prom_dw_conv", "prom_block", "prom_pack_ternary"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name


def test_pack_layout_is_as_documented(P):
    rng = np.random.default_rng(0)
    for cout, cin in ((1, 1), (3, 16), (5, 17), (7, 24), (16, 64), (9, 100)):
        w = rng.integers(-1, 2, size=(cout, cin)).astype(np.int8)
        packed = P.prom_pack_ternary(w)
        assert packed.size == P.prom_packed_size(cout, cin) == cout * ((cin + 15) // 16) * 4
        words = packed.view("<u4").reshape(cout, -1)
        for c in range(cout):
            for k in range(((cin + 15) // 16) * 16):
                e = k % 16
                d, b = e // 4, e % 4
                code = (int(words[c, k // 16]) >> (8 * b + 2 * d)) & 3
                want = 0 if k >= cin else {0: 0, 1: 1, -1: 3}[int(w[c, k])]
                assert code == want
        assert np.array_equal(P.prom_unpack_ternary(packed, cout, cin), w)


def test_pack_rejects_non_ternary_and_short_buffers(P):
    lib = P.load_library()
    w = np.zeros((4, 8), dtype=np.int8)
    w[2, 3] = 2
    with pytest.raises(P.PromError) as e:
        P.prom_pack_ternary(w)
    assert e.value.code == -6
    w[2, 3] = -1
    out = np.zeros(8, dtype=np.uint8)
    assert lib.prom_pack_ternary(w.ctypes.data, 4, 8, out.ctypes.data, 8) == -4
    assert lib.prom_pack_ternary(None, 4, 8, out.ctypes.data, 16) == -1
    assert P.prom_packed_size(0, 5) == 0 and P.prom_packed_size(5, -1) == 0


def test_strerror_covers_every_code(P):
    seen = set()
    for code in range(0, -7, -1):
        s = P.prom_strerror(code)
        assert s and "unknown" not in s
        seen.add(s)
    assert len(seen) == 7
    assert "unknown" in P.prom_strerror(-99)


def test_argument_errors_are_reported_before_any_launch(P):
    """Fake (never dereferenced) device addresses: each call must fail in host validation."""
    from paper_2505_03254_amd.binding import _RequantC
    lib = P.load_library()
    X, Wq, Y, B = 0x10000000, 0x20000000, 0x30000000, 0x40000000
    rq = _RequantC(B, B + 4096, B + 8192, 0, 127)
    r = ctypes.byref(rq)
    ok_dims = (1, 4, 4, 64)
    assert lib.prom_pw_conv(None, *ok_dims, Wq, 32, r, None, Y, None) == -1
    assert lib.prom_pw_conv(X, 0, 4, 4, 64, Wq, 32, r, None, Y, None) == -1
    assert lib.prom_pw_conv(X, *ok_dims, Wq, -3, r, None, Y, None) == -1
    assert lib.prom_pw_conv(X, *ok_dims, Wq, 32, None, None, Y, None) == -1
    assert lib.prom_pw_conv(X, *ok_dims, Wq + 2, 32, r, None, Y, None) == -1      # packed misaligned
    assert lib.prom_pw_conv(X, 1, 4, 4, 4097, Wq, 32, r, None, Y, None) == -2     # cin limit
    assert lib.prom_pw_conv(X, *ok_dims, Wq, 32, r, None, X + 512, None) == -3    # y overlaps x
    assert lib.prom_pw_conv(X, *ok_dims, Wq, 32, r, Y + 16, Y, None) == -3        # partial residual overlap
    bad = _RequantC(B, B + 4096, B + 8192, 5, 4)
    assert lib.prom_pw_conv(X, *ok_dims, Wq, 32, ctypes.byref(bad), None, Y, None) == -1
    bad = _RequantC(B, B + 4096, B + 8192, -129, 4)
    assert lib.prom_pw_conv(X, *ok_dims, Wq, 32, ctypes.byref(bad), None, Y, None) == -1
    bad = _RequantC(B, None, B + 8192, 0, 127)
    assert lib.prom_pw_conv(X, *ok_dims, Wq, 32, ctypes.byref(bad), None, Y, None) == -1
    # depthwise
    assert lib.prom_dw_conv(X, 1, 8, 8, 16, Wq, 3, r, Y, None) == -1              # stride
    assert lib.prom_dw_conv(X, 1, 8, 8, 16, None, 1, r, Y, None) == -1
    assert lib.prom_dw_conv(X, 1, 8, 8, 16, Wq, 1, r, X + 100, None) == -3
    # block
    ws = 0x50000000
    need = P.prom_block_workspace_size(1, 8, 8, 16, 96, 16, 1)
    assert need == 2 * ((8 * 8 * 96 + 255) // 256 * 256)
    args = (X, 1, 8, 8, 16, 96, 16, 1, Wq, r, Wq + 4096, r, Wq + 8192, r)
    assert lib.prom_block(*args, 1, ws, need - 1, Y, None) == -4
    assert lib.prom_block(*args, 1, None, need, Y, None) == -4
    assert lib.prom_block(*args, 1, ws + 8, need, Y, None) == -4                  # workspace alignment
    assert lib.prom_block(*args, 1, ws, need, ws + 256, None) == -3
    args2 = (X, 1, 8, 8, 16, 96, 24, 1, Wq, r, Wq + 4096, r, Wq + 8192, r)
    assert lib.prom_block(*args2, 1, ws, need, Y, None) == -1                     # residual needs cin == cout
    assert P.prom_block_workspace_size(1, 8, 8, 16, 96, 16, 3) == 0
    # grouped 3x3 and its sequence: refused before anything is enqueued, with the offending layer's index
    from paper_2505_03254_amd.binding import _GconvLayerC
    assert lib.prom_gconv3x3(X, 1, 8, 8, 16, Wq, None, 4, 3, r, Y, None) == -1      # stride
    assert lib.prom_gconv3x3(X, 1, 8, 8, 16, Wq, None, 5, 1, r, Y, None) == -1      # 16 % 5 != 0
    assert lib.prom_gconv3x3(X, 1, 8, 8, 16, Wq, None, 4, 1, r, X + 64, None) == -3  # y overlaps x
    assert lib.prom_gconv3x3(X, 1, 8, 8, 16, Wq, Wq + 8, 4, 1, r, Y, None) == -1    # prepared weights misaligned
    arr = (_GconvLayerC * 2)()
    for k in range(2):
        l = arr[k]
        l.x, l.n, l.h, l.w, l.c = X + k * 0x100000, 1, 8, 8, 16
        l.w_g, l.w_frag, l.group_size, l.stride = Wq + k * 0x1000, None, 4, 1
        l.rq, l.y = rq, Y + k * 0x100000
    arr[1].group_size = 3
    bad_layer = ctypes.c_int(-7)
    assert lib.prom_gconv3x3_sequence(arr, 2, ctypes.byref(bad_layer), None) == -1 and bad_layer.value == 1
    assert lib.prom_gconv3x3_sequence(arr, -1, None, None) == -1
    assert lib.prom_gconv3x3_sequence(None, 2, None, None) == -1
    assert lib.prom_gconv3x3_sequence(None, 0, ctypes.byref(bad_layer), None) == 0 and bad_layer.value == -1


def test_host_side_queries_of_the_launch_forms(P):
    """The planning queries run on the host alone: which form prom_block takes, where the two
    one-kernel forms apply, and where prom_pw_conv takes the kernel for wide layers."""
    # plane-resident block kernel: hidden channels a multiple of 16, cin % 8 == 0 and <= 192, cout % 4 == 0
    assert P.prom_block_planes_applies(128, 14, 14, 64, 384, 64, 1)
    assert P.prom_block_planes_applies(1, 1, 1, 8, 16, 4, 1)
    assert P.prom_block_planes_applies(2, 7, 7, 160, 960, 320, 2)
    assert not P.prom_block_planes_applies(2, 7, 7, 12, 72, 16, 1)        # cin % 8
    assert not P.prom_block_planes_applies(2, 7, 7, 16, 72, 16, 1)        # hidden % 16
    assert not P.prom_block_planes_applies(2, 7, 7, 16, 96, 18, 1)        # cout % 4
    assert not P.prom_block_planes_applies(2, 7, 7, 200, 1600, 200, 1)    # cin > 192
    assert not P.prom_block_planes_applies(1, 4, 6000, 16, 96, 16, 1)     # rows wider than the kernel takes
    with pytest.raises(P.PromError):
        P.prom_block_planes_applies(0, 7, 7, 16, 96, 16, 1)
    with pytest.raises(P.PromError):
        P.prom_block_planes_applies(1, 7, 7, 16, 96, 16, 3)
    # what prom_block picks: one kernel for deep blocks on small maps and for small problems
    assert P.prom_block_is_fused(128, 14, 14, 96, 576, 96, 1)
    assert P.prom_block_is_fused(8, 112, 112, 16, 96, 24, 2)
    assert not P.prom_block_is_fused(128, 56, 56, 24, 144, 24, 1)
    assert not P.prom_block_is_fused(4, 14, 14, 60, 360, 60, 1)
    # pointwise plans: the kernel for wide layers from 1024 input and 256 output channels on
    q = P.prom_pw_plan_query(128, 7, 7, 2048, 1024)
    assert q["k_outer"] == 1
    assert P.prom_pw_plan_query(128, 7, 7, 1024, 128)["k_outer"] == 0
    assert P.prom_pw_plan_query(128, 14, 14, 960, 320)["k_outer"] == 0
    assert P.prom_pw_plan_query(128, 14, 14, 1032, 512)["k_outer"] == 0   # cin % 64
    # ... when its tiles fill the chip (tiles x k steps >= 2800)
    assert P.prom_pw_plan_query(32, 7, 7, 2048, 1024)["k_outer"] == 0      # 56 tiles of 32 k steps
    assert P.prom_pw_plan_query(32, 14, 14, 1024, 1024)["k_outer"] == 1    # 200 tiles of 16
    assert P.prom_pw_plan_query(64, 7, 7, 2048, 1024)["k_outer"] == 1      # 104 tiles of 32
    # layers that take the kernel for wide layers never join a shared launch
    assert P.prom_pw_batch_class(128, 7, 7, 2048, 1024) == 0


def test_binding_fails_loudly_without_library(P, monkeypatch):
    import paper_2505_03254_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libprom.so")
    with pytest.raises(RuntimeError):
        b.load_library()
