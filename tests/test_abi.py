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


def test_binding_fails_loudly_without_library(P, monkeypatch):
    import paper_2505_03254_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libprom.so")
    with pytest.raises(RuntimeError):
        b.load_library()
