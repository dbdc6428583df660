"""ctypes loader for the plain-C oracle (oracle/prom_oracle.c).

Test infrastructure only.  Builds libprom_oracle.so with gcc next to this file on
first use (or when build() is called) and wraps each C function for numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "prom_oracle.c")
_LIB = os.path.join(_HERE, "libprom_oracle.so")
_lib = None

_i8p = ctypes.POINTER(ctypes.c_int8)
_i32p = ctypes.POINTER(ctypes.c_int32)


def build(force: bool = True) -> str:
    """Compile the oracle with gcc -O2 -fopenmp.  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        lib.oracle_requant.restype = ctypes.c_int64
        lib.oracle_requant.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        lib.oracle_max_threads.restype = ctypes.c_int
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        lib.oracle_pw_accum.restype = ctypes.c_int
        lib.oracle_pw_accum.argtypes = [_i8p, ctypes.c_int64, ctypes.c_int, _i8p, ctypes.c_int, _i32p]
        lib.oracle_pw_conv.restype = ctypes.c_int
        lib.oracle_pw_conv.argtypes = [_i8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       _i8p, ctypes.c_int, _i32p, _i32p, _i32p,
                                       ctypes.c_int32, ctypes.c_int32, _i8p, _i8p]
        lib.oracle_dw_conv.restype = ctypes.c_int
        lib.oracle_dw_conv.argtypes = [_i8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                       _i8p, ctypes.c_int, _i32p, _i32p, _i32p,
                                       ctypes.c_int32, ctypes.c_int32, _i8p]
        lib.oracle_requant_prelu.restype = ctypes.c_int64
        lib.oracle_requant_prelu.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        lib.oracle_pw_conv_prelu.restype = ctypes.c_int
        lib.oracle_pw_conv_prelu.argtypes = [_i8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                             _i8p, ctypes.c_int, _i32p, _i32p, _i32p, _i32p,
                                             ctypes.c_int32, ctypes.c_int32, _i8p, _i8p]
        lib.oracle_dw_conv_prelu.restype = ctypes.c_int
        lib.oracle_dw_conv_prelu.argtypes = [_i8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                             _i8p, ctypes.c_int, _i32p, _i32p, _i32p, _i32p,
                                             ctypes.c_int32, ctypes.c_int32, _i8p]
        lib.oracle_gconv3x3.restype = ctypes.c_int
        lib.oracle_gconv3x3.argtypes = [_i8p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                        _i8p, ctypes.c_int, ctypes.c_int, _i32p, _i32p, _i32p, _i32p,
                                        ctypes.c_int32, ctypes.c_int32, _i32p, _i8p]
        lib.oracle_block.restype = ctypes.c_int
        lib.oracle_block.argtypes = ([_i8p] + [ctypes.c_int] * 7 +
                                     [_i8p, _i32p, _i32p, _i32p, ctypes.c_int32, ctypes.c_int32] * 3 +
                                     [ctypes.c_int, _i8p, _i8p, _i8p])
        _lib = lib
    return _lib


def _i8(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.int8)
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p8(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_i8p)


def _p32(a: np.ndarray):
    return a.ctypes.data_as(_i32p)


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(int(n))


def requant(s: int, mult: int, shift: int) -> int:
    return int(_load().oracle_requant(int(s), int(mult), int(shift)))


def requant_prelu(s: int, mult: int, mult_neg: int, shift: int) -> int:
    return int(_load().oracle_requant_prelu(int(s), int(mult), int(mult_neg), int(shift)))


def pw_accum(x: np.ndarray, weight: np.ndarray) -> np.ndarray:
    """x int8 [..., cin], weight int8 [cout, cin] -> int32 [..., cout]."""
    x = _i8(x)
    weight = _i8(weight)
    cout, cin = weight.shape
    m = x.size // cin
    acc = np.empty(x.shape[:-1] + (cout,), dtype=np.int32)
    rc = _load().oracle_pw_accum(_p8(x), m, cin, _p8(weight), cout, _p32(acc))
    if rc:
        raise ValueError(f"oracle_pw_accum failed: {rc}")
    return acc


def pw_conv(x, weight, bias, mult, shift, act_min: int, act_max: int,
            residual=None, mult_neg=None) -> np.ndarray:
    """x int8 [n,h,w,cin]; weight int8 [cout,cin] ternary -> int8 [n,h,w,cout].
    With mult_neg (int32 [cout]) the PReLU requantisation is used."""
    x = _i8(x)
    weight = _i8(weight)
    n, h, w, cin = x.shape
    cout = weight.shape[0]
    assert weight.shape == (cout, cin)
    bias, mult, shift = _i32(bias), _i32(mult), _i32(shift)
    assert bias.shape == mult.shape == shift.shape == (cout,)
    res = None
    if residual is not None:
        res = _i8(residual)
        assert res.shape == (n, h, w, cout)
    y = np.empty((n, h, w, cout), dtype=np.int8)
    if mult_neg is not None:
        mult_neg = _i32(mult_neg)
        assert mult_neg.shape == (cout,)
        rc = _load().oracle_pw_conv_prelu(_p8(x), n, h, w, cin, _p8(weight), cout, _p32(bias),
                                          _p32(mult), _p32(mult_neg), _p32(shift), act_min, act_max,
                                          _p8(res), _p8(y))
        if rc:
            raise ValueError(f"oracle_pw_conv_prelu failed: {rc}")
        return y
    rc = _load().oracle_pw_conv(_p8(x), n, h, w, cin, _p8(weight), cout, _p32(bias), _p32(mult),
                                _p32(shift), act_min, act_max, _p8(res), _p8(y))
    if rc:
        raise ValueError(f"oracle_pw_conv failed: {rc}")
    return y


def dw_conv(x, weight, stride: int, bias, mult, shift, act_min: int, act_max: int,
            mult_neg=None) -> np.ndarray:
    """x int8 [n,h,w,c]; weight int8 [3,3,c] -> int8 [n,ho,wo,c] (pad 1).
    With mult_neg (int32 [c]) the PReLU requantisation is used."""
    x = _i8(x)
    weight = _i8(weight)
    n, h, w, c = x.shape
    assert weight.shape == (3, 3, c)
    bias, mult, shift = _i32(bias), _i32(mult), _i32(shift)
    ho = (h + 2 - 3) // stride + 1
    wo = (w + 2 - 3) // stride + 1
    y = np.empty((n, ho, wo, c), dtype=np.int8)
    if mult_neg is not None:
        mult_neg = _i32(mult_neg)
        assert mult_neg.shape == (c,)
        rc = _load().oracle_dw_conv_prelu(_p8(x), n, h, w, c, _p8(weight), stride, _p32(bias),
                                          _p32(mult), _p32(mult_neg), _p32(shift), act_min, act_max,
                                          _p8(y))
        if rc:
            raise ValueError(f"oracle_dw_conv_prelu failed: {rc}")
        return y
    rc = _load().oracle_dw_conv(_p8(x), n, h, w, c, _p8(weight), stride, _p32(bias), _p32(mult),
                                _p32(shift), act_min, act_max, _p8(y))
    if rc:
        raise ValueError(f"oracle_dw_conv failed: {rc}")
    return y


def _gconv(x, weight, stride, bias, mult, mult_neg, shift, act_min, act_max, raw):
    x = _i8(x)
    weight = _i8(weight)
    n, h, w, c = x.shape
    assert weight.ndim == 4 and weight.shape[:3] == (3, 3, c), weight.shape
    gs = weight.shape[3]
    ho = (h + 2 - 3) // stride + 1
    wo = (w + 2 - 3) // stride + 1
    null32 = ctypes.cast(None, _i32p)
    if raw:
        acc = np.empty((n, ho, wo, c), dtype=np.int32)
        rc = _load().oracle_gconv3x3(_p8(x), n, h, w, c, _p8(weight), gs, stride, null32, null32, null32,
                                     null32, 0, 0, _p32(acc), None)
        out = acc
    else:
        bias, mult, shift = _i32(bias), _i32(mult), _i32(shift)
        assert bias.shape == mult.shape == shift.shape == (c,)
        mn = null32
        if mult_neg is not None:
            mult_neg = _i32(mult_neg)
            assert mult_neg.shape == (c,)
            mn = _p32(mult_neg)
        y = np.empty((n, ho, wo, c), dtype=np.int8)
        rc = _load().oracle_gconv3x3(_p8(x), n, h, w, c, _p8(weight), gs, stride, _p32(bias), _p32(mult), mn,
                                     _p32(shift), act_min, act_max, null32, _p8(y))
        out = y
    if rc:
        raise ValueError(f"oracle_gconv3x3 failed: {rc}")
    return out


def gconv3x3(x, weight, stride: int, bias, mult, shift, act_min: int, act_max: int,
             mult_neg=None) -> np.ndarray:
    """Grouped 3x3 conv: x int8 [n,h,w,c]; weight int8 [3,3,c,gs] -> int8 [n,ho,wo,c] (pad 1)."""
    return _gconv(x, weight, stride, bias, mult, mult_neg, shift, act_min, act_max, False)


def gconv3x3_accum(x, weight, stride: int) -> np.ndarray:
    """Raw int32 sums of the grouped 3x3 conv."""
    return _gconv(x, weight, stride, None, None, None, None, 0, 0, True)


def block(x, expand, dw, project, stride: int, add_residual: bool):
    """expand/dw/project are tuples (weight, bias, mult, shift, act_min, act_max).
    Returns (y, t1, t2) with the two intermediates."""
    x = _i8(x)
    n, h, w, cin = x.shape
    we, be, me, se, loe, hie = expand
    wd_, bd, md, sd, lod, hid = dw
    wp, bp, mp, sp, lop, hip_ = project
    we, wd_, wp = _i8(we), _i8(wd_), _i8(wp)
    chid = we.shape[0]
    cout = wp.shape[0]
    ho = (h + 2 - 3) // stride + 1
    wo = (w + 2 - 3) // stride + 1
    t1 = np.empty((n, h, w, chid), dtype=np.int8)
    t2 = np.empty((n, ho, wo, chid), dtype=np.int8)
    y = np.empty((n, ho, wo, cout), dtype=np.int8)
    be, me, se = _i32(be), _i32(me), _i32(se)
    bd, md, sd = _i32(bd), _i32(md), _i32(sd)
    bp, mp, sp = _i32(bp), _i32(mp), _i32(sp)
    rc = _load().oracle_block(_p8(x), n, h, w, cin, chid, cout, stride,
                              _p8(we), _p32(be), _p32(me), _p32(se), loe, hie,
                              _p8(wd_), _p32(bd), _p32(md), _p32(sd), lod, hid,
                              _p8(wp), _p32(bp), _p32(mp), _p32(sp), lop, hip_,
                              int(bool(add_residual)), _p8(t1), _p8(t2), _p8(y))
    if rc:
        raise ValueError(f"oracle_block failed: {rc}")
    return y, t1, t2


def block_prelu(x, expand, dw, project, stride: int, add_residual: bool):
    """The block with PReLU after the expand and depthwise layers (the paper's MobileNetV2
    variant, Section 3.2): the three layer functions chained.  expand and dw are tuples
    (weight, bias, mult, shift, act_min, act_max, mult_neg); project as in block()."""
    we, be, me, se, loe, hie, ne = expand
    wd_, bd, md, sd, lod, hid, nd = dw
    wp, bp, mp, sp, lop, hip_ = project
    t1 = pw_conv(x, we, be, me, se, loe, hie, mult_neg=ne)
    t2 = dw_conv(t1, wd_, stride, bd, md, sd, lod, hid, mult_neg=nd)
    y = pw_conv(t2, wp, bp, mp, sp, lop, hip_, residual=_i8(x) if add_residual else None)
    return y, t1, t2
