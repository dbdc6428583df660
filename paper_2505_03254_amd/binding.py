"""ctypes binding of include/prom.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libprom.so")
_lib = None

PROM_OK = 0


class PromError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        detail = ""
        if code == -5:
            detail = " [" + load_library().prom_last_hip_error().decode() + "]"
        super().__init__(f"{where}: {prom_strerror(code)} (code {code}){detail}")


class _RequantC(ctypes.Structure):
    _fields_ = [("bias", ctypes.c_void_p), ("mult", ctypes.c_void_p), ("shift", ctypes.c_void_p),
                ("act_min", ctypes.c_int32), ("act_max", ctypes.c_int32),
                ("mult_neg", ctypes.c_void_p)]


class _PwLayerC(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("n", ctypes.c_int32), ("h", ctypes.c_int32),
                ("w", ctypes.c_int32), ("cin", ctypes.c_int32), ("w_packed", ctypes.c_void_p),
                ("cout", ctypes.c_int32), ("rq", _RequantC), ("residual", ctypes.c_void_p),
                ("y", ctypes.c_void_p)]


class _DwLayerC(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("n", ctypes.c_int32), ("h", ctypes.c_int32),
                ("w", ctypes.c_int32), ("c", ctypes.c_int32), ("w_dw", ctypes.c_void_p),
                ("stride", ctypes.c_int32), ("rq", _RequantC), ("y", ctypes.c_void_p)]


class _GconvLayerC(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("n", ctypes.c_int32), ("h", ctypes.c_int32),
                ("w", ctypes.c_int32), ("c", ctypes.c_int32), ("w_g", ctypes.c_void_p),
                ("w_frag", ctypes.c_void_p), ("group_size", ctypes.c_int32), ("stride", ctypes.c_int32),
                ("rq", _RequantC), ("y", ctypes.c_void_p)]


class _PlanC(ctypes.Structure):
    _fields_ = [("tiles_per_wave", ctypes.c_int32), ("pixel_tiles", ctypes.c_int32),
                ("workgroups", ctypes.c_int32), ("row_waves", ctypes.c_int32), ("k_outer", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libprom.so; raises if it has not been built (there is no CPU fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                           f"`python -m paper_2505_03254_amd.build` (needs hipcc)")
    # The process must hold ONE HIP runtime.  PyTorch ships its own libamdhip64 (same
    # soname as the system one); importing torch first makes the dynamic loader bind
    # libprom.so to that copy, so kernels launch on the runtime that owns torch's device
    # memory and streams.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.prom_packed_size.restype = sz
    lib.prom_packed_size.argtypes = [ci, ci]
    lib.prom_pack_ternary.restype = ci
    lib.prom_pack_ternary.argtypes = [vp, ci, ci, vp, sz]
    lib.prom_unpack_ternary.restype = ci
    lib.prom_unpack_ternary.argtypes = [vp, sz, ci, ci, vp]
    lib.prom_pw_conv.restype = ci
    lib.prom_pw_conv.argtypes = [vp, ci, ci, ci, ci, vp, ci, ctypes.POINTER(_RequantC), vp, vp, vp]
    lib.prom_pw_conv_addsub.restype = ci
    lib.prom_pw_conv_addsub.argtypes = [vp, ci, ci, ci, ci, vp, ci, ctypes.POINTER(_RequantC), vp, vp, vp]
    lib.prom_pw_conv_ex.restype = ci
    lib.prom_pw_conv_ex.argtypes = [vp, ci, ci, ci, ci, vp, ci, ctypes.POINTER(_RequantC), vp, vp,
                                    ctypes.POINTER(_PlanC), vp]
    lib.prom_pw_accum_i32.restype = ci
    lib.prom_pw_accum_i32.argtypes = [vp, ci, ci, ci, ci, vp, ci, vp, vp]
    lib.prom_dw_conv.restype = ci
    lib.prom_dw_conv.argtypes = [vp, ci, ci, ci, ci, vp, ci, ctypes.POINTER(_RequantC), vp, vp]
    lib.prom_gconv3x3.restype = ci
    lib.prom_gconv3x3.argtypes = [vp, ci, ci, ci, ci, vp, vp, ci, ci, ctypes.POINTER(_RequantC), vp, vp]
    lib.prom_gconv_frag_size.restype = sz
    lib.prom_gconv_frag_size.argtypes = [ci, ci]
    lib.prom_gconv_pack.restype = ci
    lib.prom_gconv_pack.argtypes = [vp, ci, ci, vp, sz]
    lib.prom_block.restype = ci
    lib.prom_block.argtypes = [vp, ci, ci, ci, ci, ci, ci, ci,
                               vp, ctypes.POINTER(_RequantC), vp, ctypes.POINTER(_RequantC),
                               vp, ctypes.POINTER(_RequantC), ci, vp, sz, vp, vp]
    lib.prom_block_ex.restype = ci
    lib.prom_block_ex.argtypes = [vp, ci, ci, ci, ci, ci, ci, ci,
                                  vp, ctypes.POINTER(_RequantC), vp, ctypes.POINTER(_RequantC),
                                  vp, ctypes.POINTER(_RequantC), ci, vp, sz, vp, ci, vp]
    lib.prom_block_noalloc.restype = ci
    lib.prom_block_noalloc.argtypes = [vp, ci, ci, ci, ci, ci, ci, ci,
                                       vp, ctypes.POINTER(_RequantC), vp, ctypes.POINTER(_RequantC),
                                       vp, ctypes.POINTER(_RequantC), ci, vp, vp]
    lib.prom_block_noalloc_max_workspace.restype = sz
    lib.prom_block_noalloc_max_workspace.argtypes = []
    lib.prom_dw_pw_conv.restype = ci
    lib.prom_dw_pw_conv.argtypes = [vp, ci, ci, ci, ci, vp, ci, ctypes.POINTER(_RequantC), vp, ci,
                                    ctypes.POINTER(_RequantC), vp, vp, vp]
    lib.prom_dw_pw_can_fuse.restype = ci
    lib.prom_dw_pw_can_fuse.argtypes = [ci] * 6
    lib.prom_block_can_fuse.restype = ci
    lib.prom_block_can_fuse.argtypes = [ci] * 7
    lib.prom_block_planes_applies.restype = ci
    lib.prom_block_planes_applies.argtypes = [ci] * 7
    lib.prom_block_workspace_size.restype = sz
    lib.prom_block_workspace_size.argtypes = [ci] * 7
    lib.prom_pw_plan_query.restype = ci
    lib.prom_pw_plan_query.argtypes = [ci, ci, ci, ci, ci, ctypes.POINTER(_PlanC), ctypes.POINTER(ci)]
    lib.prom_pw_conv_sequence.restype = ci
    lib.prom_pw_conv_sequence.argtypes = [ctypes.POINTER(_PwLayerC), ci, ctypes.POINTER(ci), vp]
    lib.prom_dw_conv_sequence.restype = ci
    lib.prom_dw_conv_sequence.argtypes = [ctypes.POINTER(_DwLayerC), ci, ctypes.POINTER(ci), vp]
    lib.prom_gconv3x3_sequence.restype = ci
    lib.prom_gconv3x3_sequence.argtypes = [ctypes.POINTER(_GconvLayerC), ci, ctypes.POINTER(ci), vp]
    lib.prom_quantize_pw_absmean.restype = ci
    lib.prom_quantize_pw_absmean.argtypes = [vp, ci, ci, ctypes.c_float, vp, sz, vp, vp, vp]
    lib.prom_quantize_activation_absmax.restype = ci
    lib.prom_quantize_activation_absmax.argtypes = [vp, ci, ctypes.c_longlong, ctypes.c_float, vp, vp, vp]
    lib.prom_pw_conv_dynq.restype = ci
    lib.prom_pw_conv_dynq.argtypes = [vp, ci, ci, ci, ci, vp, ci, vp, vp, vp, ci, ctypes.c_float, vp, vp, vp, vp]
    lib.prom_quantize_dw_absmax.restype = ci
    lib.prom_quantize_dw_absmax.argtypes = [vp, ci, ctypes.c_float, vp, vp, vp]
    lib.prom_quantize_gconv_absmax.restype = ci
    lib.prom_quantize_gconv_absmax.argtypes = [vp, ci, ci, ctypes.c_float, vp, vp, vp]
    lib.prom_block_is_fused.restype = ci
    lib.prom_block_is_fused.argtypes = [ci] * 7
    lib.prom_pw_batch_class.restype = ci
    lib.prom_pw_batch_class.argtypes = [ci, ci, ci, ci, ci]
    lib.prom_pw_batchable.restype = ci
    lib.prom_pw_batchable.argtypes = [ci, ci, ci, ci, ci]
    lib.prom_copy_bytes.restype = ci
    lib.prom_copy_bytes.argtypes = [vp, vp, sz, vp]
    lib.prom_stream_read.restype = ci
    lib.prom_stream_read.argtypes = [vp, sz, vp, vp]
    lib.prom_stream_write.restype = ci
    lib.prom_stream_write.argtypes = [vp, sz, ci, vp]
    lib.prom_mfma_i8_loop.restype = ctypes.c_longlong
    lib.prom_mfma_i8_loop.argtypes = [ci, vp, vp]
    lib.prom_requant_check.restype = ci
    lib.prom_requant_check.argtypes = [ctypes.POINTER(_RequantC), ci, ci, ctypes.POINTER(ci)]
    lib.prom_strerror.restype = ctypes.c_char_p
    lib.prom_strerror.argtypes = [ci]
    lib.prom_last_hip_error.restype = ctypes.c_char_p
    lib.prom_last_hip_error.argtypes = []
    _lib = lib
    return lib


def prom_strerror(code: int) -> str:
    return load_library().prom_strerror(int(code)).decode()


def _check(rc: int, where: str) -> None:
    if rc != PROM_OK:
        raise PromError(rc, where)


@dataclass
class Requant:
    """Device int32 tensors bias/mult/shift of one layer plus its activation window;
    mult_neg (optional) makes it a PReLU layer."""
    bias: "torch.Tensor"
    mult: "torch.Tensor"
    shift: "torch.Tensor"
    act_min: int
    act_max: int
    mult_neg: "Optional[torch.Tensor]" = None

    def _c(self) -> _RequantC:
        import torch
        for t in (self.bias, self.mult, self.shift) + (() if self.mult_neg is None else (self.mult_neg,)):
            assert t.dtype == torch.int32 and t.is_contiguous() and t.is_cuda
        if self.mult_neg is not None:
            assert self.mult_neg.numel() == self.mult.numel()
        return _RequantC(self.bias.data_ptr(), self.mult.data_ptr(), self.shift.data_ptr(),
                         int(self.act_min), int(self.act_max),
                         None if self.mult_neg is None else self.mult_neg.data_ptr())


@dataclass
class PwPlan:
    tiles_per_wave: int = 0
    pixel_tiles: int = 0
    workgroups: int = 0
    row_waves: int = 0
    k_outer: int = 0

    def _c(self) -> _PlanC:
        return _PlanC(self.tiles_per_wave, self.pixel_tiles, self.workgroups, self.row_waves, self.k_outer)


def _stream_ptr(stream) -> int:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev_i8(t, name):
    import torch
    if not (t.is_cuda and t.dtype == torch.int8 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous int8 device tensor")
    return t


# ---- host-side packing --------------------------------------------------------------------
def prom_packed_size(cout: int, cin: int) -> int:
    return int(load_library().prom_packed_size(int(cout), int(cin)))


def prom_pack_ternary(w: np.ndarray) -> np.ndarray:
    """w: int8 [cout][cin] host array with values in {-1,0,1} -> packed bytes (uint8 host array)."""
    w = np.ascontiguousarray(w, dtype=np.int8)
    cout, cin = w.shape
    out = np.zeros(prom_packed_size(cout, cin), dtype=np.uint8)
    rc = load_library().prom_pack_ternary(w.ctypes.data, cout, cin, out.ctypes.data, out.size)
    _check(rc, "prom_pack_ternary")
    return out


def prom_unpack_ternary(packed: np.ndarray, cout: int, cin: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    w = np.empty((cout, cin), dtype=np.int8)
    rc = load_library().prom_unpack_ternary(packed.ctypes.data, packed.size, cout, cin, w.ctypes.data)
    _check(rc, "prom_unpack_ternary")
    return w


# ---- device entry points --------------------------------------------------------------------
def prom_pw_conv_ex(x, w_packed, cout: int, rq: Requant, residual=None, y=None,
                    plan: Optional[PwPlan] = None, stream=None):
    """x: int8 [n,h,w,cin] device; w_packed: uint8 device tensor from prom_pack_ternary."""
    import torch
    _dev_i8(x, "x")
    n, h, w, cin = x.shape
    if y is None:
        y = torch.empty((n, h, w, cout), dtype=torch.int8, device=x.device)
    _dev_i8(y, "y")
    if residual is not None:
        _dev_i8(residual, "residual")
    rqc = rq._c()
    planc = plan._c() if plan is not None else None
    rc = load_library().prom_pw_conv_ex(
        x.data_ptr(), n, h, w, cin, w_packed.data_ptr(), int(cout), ctypes.byref(rqc),
        residual.data_ptr() if residual is not None else None, y.data_ptr(),
        ctypes.byref(planc) if planc is not None else None, _stream_ptr(stream))
    _check(rc, "prom_pw_conv_ex")
    return y


def prom_pw_conv(x, w_packed, cout: int, rq: Requant, residual=None, y=None, stream=None):
    import torch
    _dev_i8(x, "x")
    n, h, w, cin = x.shape
    if y is None:
        y = torch.empty((n, h, w, cout), dtype=torch.int8, device=x.device)
    _dev_i8(y, "y")
    if residual is not None:
        _dev_i8(residual, "residual")
    rqc = rq._c()
    rc = load_library().prom_pw_conv(
        x.data_ptr(), n, h, w, cin, w_packed.data_ptr(), int(cout), ctypes.byref(rqc),
        residual.data_ptr() if residual is not None else None, y.data_ptr(), _stream_ptr(stream))
    _check(rc, "prom_pw_conv")
    return y


def prom_pw_conv_addsub(x, w_packed, cout: int, rq: Requant, residual=None, y=None, stream=None):
    """The add/subtract (vector ALU) design of the same layer, for the A/B measurement."""
    import torch
    _dev_i8(x, "x")
    n, h, w, cin = x.shape
    if y is None:
        y = torch.empty((n, h, w, cout), dtype=torch.int8, device=x.device)
    _dev_i8(y, "y")
    if residual is not None:
        _dev_i8(residual, "residual")
    rqc = rq._c()
    rc = load_library().prom_pw_conv_addsub(
        x.data_ptr(), n, h, w, cin, w_packed.data_ptr(), int(cout), ctypes.byref(rqc),
        residual.data_ptr() if residual is not None else None, y.data_ptr(), _stream_ptr(stream))
    _check(rc, "prom_pw_conv_addsub")
    return y


def prom_pw_accum_i32(x, w_packed, cout: int, acc=None, stream=None):
    import torch
    _dev_i8(x, "x")
    n, h, w, cin = x.shape
    if acc is None:
        acc = torch.empty((n, h, w, cout), dtype=torch.int32, device=x.device)
    rc = load_library().prom_pw_accum_i32(x.data_ptr(), n, h, w, cin, w_packed.data_ptr(), int(cout),
                                          acc.data_ptr(), _stream_ptr(stream))
    _check(rc, "prom_pw_accum_i32")
    return acc


def prom_dw_conv(x, w_dw, stride: int, rq: Requant, y=None, stream=None):
    """x: int8 [n,h,w,c] device; w_dw: int8 [3,3,c] device."""
    import torch
    _dev_i8(x, "x")
    _dev_i8(w_dw, "w_dw")
    n, h, w, c = x.shape
    ho, wo = (h - 1) // stride + 1, (w - 1) // stride + 1
    if y is None:
        y = torch.empty((n, ho, wo, c), dtype=torch.int8, device=x.device)
    _dev_i8(y, "y")
    rqc = rq._c()
    rc = load_library().prom_dw_conv(x.data_ptr(), n, h, w, c, w_dw.data_ptr(), int(stride),
                                     ctypes.byref(rqc), y.data_ptr(), _stream_ptr(stream))
    _check(rc, "prom_dw_conv")
    return y


def prom_block_workspace_size(n, h, w, cin, chid, cout, stride) -> int:
    return int(load_library().prom_block_workspace_size(n, h, w, cin, chid, cout, stride))


def prom_gconv_frag_size(c: int, group_size: int) -> int:
    return int(load_library().prom_gconv_frag_size(int(c), int(group_size)))


def prom_gconv_pack(w: np.ndarray) -> np.ndarray:
    """w: int8 [3,3,c,group_size] host array -> the prepared form for the matrix-core kernel
    (uint8 host array).  Raises PromError(-2) when that kernel does not take the layer."""
    w = np.ascontiguousarray(w, dtype=np.int8)
    assert w.ndim == 4 and w.shape[:2] == (3, 3)
    c, gs = int(w.shape[2]), int(w.shape[3])
    out = np.zeros(max(prom_gconv_frag_size(c, gs), 1), dtype=np.uint8)
    _check(load_library().prom_gconv_pack(w.ctypes.data, c, gs, out.ctypes.data, out.size), "prom_gconv_pack")
    return out


def prom_gconv3x3(x, w_g, stride: int, rq: Requant, y=None, stream=None, w_frag=None):
    """Grouped 3x3 conv: x int8 [n,h,w,c] device; w_g int8 [3,3,c,group_size] device;
    w_frag: optional device copy of prom_gconv_pack(w_g)."""
    import torch
    _dev_i8(x, "x")
    _dev_i8(w_g, "w_g")
    n, h, w, c = x.shape
    if w_g.dim() != 4 or tuple(w_g.shape[:3]) != (3, 3, c):
        raise ValueError("w_g must have the shape [3, 3, c, group_size]")
    gs = int(w_g.shape[3])
    ho, wo = (h - 1) // stride + 1, (w - 1) // stride + 1
    if y is None:
        y = torch.empty((n, ho, wo, c), dtype=torch.int8, device=x.device)
    _dev_i8(y, "y")
    rqc = rq._c()
    _check(load_library().prom_gconv3x3(x.data_ptr(), n, h, w, c, w_g.data_ptr(),
                                        None if w_frag is None else w_frag.data_ptr(), gs, int(stride),
                                        ctypes.byref(rqc), y.data_ptr(), _stream_ptr(stream)), "prom_gconv3x3")
    return y


def prom_block(x, chid: int, cout: int, stride: int, w_expand_packed, rq_expand: Requant,
               w_dw, rq_dw: Requant, w_project_packed, rq_project: Requant, add_residual: bool,
               workspace, y=None, stream=None, path: int = 0):
    """path: BLOCK_AUTO (0, the library picks), BLOCK_FUSED (1) or BLOCK_UNFUSED (2): prom_block_ex."""
    import torch
    _dev_i8(x, "x")
    _dev_i8(w_dw, "w_dw")
    n, h, w, cin = x.shape
    ho, wo = (h - 1) // stride + 1, (w - 1) // stride + 1
    if y is None:
        y = torch.empty((n, ho, wo, cout), dtype=torch.int8, device=x.device)
    _dev_i8(y, "y")
    e, d, p = rq_expand._c(), rq_dw._c(), rq_project._c()
    rc = load_library().prom_block_ex(
        x.data_ptr(), n, h, w, cin, int(chid), int(cout), int(stride),
        w_expand_packed.data_ptr(), ctypes.byref(e), w_dw.data_ptr(), ctypes.byref(d),
        w_project_packed.data_ptr(), ctypes.byref(p), int(bool(add_residual)),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), y.data_ptr(),
        int(path), _stream_ptr(stream))
    _check(rc, "prom_block")
    return y


BLOCK_AUTO, BLOCK_FUSED, BLOCK_UNFUSED, BLOCK_DWPROJ, BLOCK_PLANES = 0, 1, 2, 3, 4


def prom_dw_pw_conv(x, w_dw, stride: int, rq_dw: Requant, w_project_packed, cout: int, rq_project: Requant,
                    residual=None, y=None, stream=None):
    """Depthwise 3x3 and the pointwise projection behind it in one kernel."""
    import torch
    _dev_i8(x, "x")
    _dev_i8(w_dw, "w_dw")
    n, h, w, c = x.shape
    ho, wo = (h - 1) // stride + 1, (w - 1) // stride + 1
    if y is None:
        y = torch.empty((n, ho, wo, cout), dtype=torch.int8, device=x.device)
    _dev_i8(y, "y")
    if residual is not None:
        _dev_i8(residual, "residual")
    d, p = rq_dw._c(), rq_project._c()
    rc = load_library().prom_dw_pw_conv(
        x.data_ptr(), n, h, w, c, w_dw.data_ptr(), int(stride), ctypes.byref(d), w_project_packed.data_ptr(),
        int(cout), ctypes.byref(p), residual.data_ptr() if residual is not None else None, y.data_ptr(),
        _stream_ptr(stream))
    _check(rc, "prom_dw_pw_conv")
    return y


def prom_dw_pw_can_fuse(n: int, h: int, w: int, c: int, cout: int, stride: int) -> bool:
    rc = load_library().prom_dw_pw_can_fuse(n, h, w, c, cout, stride)
    if rc < 0:
        raise PromError(rc, "prom_dw_pw_can_fuse")
    return bool(rc)


def prom_block_noalloc(x, chid: int, cout: int, stride: int, w_expand_packed, rq_expand: Requant,
                       w_dw, rq_dw: Requant, w_project_packed, rq_project: Requant, add_residual: bool,
                       y, stream=None):
    """prom_block without a workspace: the intermediates live in the library's fixed device array.
    The caller passes the output tensor (nothing is allocated here either)."""
    _dev_i8(x, "x")
    _dev_i8(w_dw, "w_dw")
    _dev_i8(y, "y")
    n, h, w, cin = x.shape
    e, d, p = rq_expand._c(), rq_dw._c(), rq_project._c()
    rc = load_library().prom_block_noalloc(
        x.data_ptr(), n, h, w, cin, int(chid), int(cout), int(stride),
        w_expand_packed.data_ptr(), ctypes.byref(e), w_dw.data_ptr(), ctypes.byref(d),
        w_project_packed.data_ptr(), ctypes.byref(p), int(bool(add_residual)), y.data_ptr(),
        _stream_ptr(stream))
    _check(rc, "prom_block_noalloc")
    return y


def prom_block_noalloc_max_workspace() -> int:
    return int(load_library().prom_block_noalloc_max_workspace())


def prom_block_planes_applies(n: int, h: int, w: int, cin: int, chid: int, cout: int, stride: int) -> bool:
    rc = load_library().prom_block_planes_applies(n, h, w, cin, chid, cout, stride)
    if rc < 0:
        raise PromError(rc, "prom_block_planes_applies")
    return bool(rc)


def prom_block_can_fuse(n: int, h: int, w: int, cin: int, chid: int, cout: int, stride: int) -> bool:
    rc = load_library().prom_block_can_fuse(n, h, w, cin, chid, cout, stride)
    if rc < 0:
        raise PromError(rc, "prom_block_can_fuse")
    return bool(rc)


def prom_quantize_pw_absmean(w, eps: float = 1e-5, want_codes: bool = False, stream=None):
    """w: float32 [cout, cin] device.  Returns (packed uint8 device tensor in the prom_pack_ternary
    layout, scale float32 [cout], codes int8 [cout, cin] or None)."""
    import torch
    if not (w.is_cuda and w.dtype == torch.float32 and w.is_contiguous() and w.dim() == 2):
        raise TypeError("w must be a contiguous float32 [cout, cin] device tensor")
    cout, cin = w.shape
    nbytes = prom_packed_size(cout, cin)
    packed = torch.empty(nbytes, dtype=torch.uint8, device=w.device)
    scale = torch.empty(cout, dtype=torch.float32, device=w.device)
    codes = torch.empty((cout, cin), dtype=torch.int8, device=w.device) if want_codes else None
    _check(load_library().prom_quantize_pw_absmean(
        w.data_ptr(), cout, cin, float(eps), packed.data_ptr(), nbytes,
        codes.data_ptr() if codes is not None else None, scale.data_ptr(), _stream_ptr(stream)),
        "prom_quantize_pw_absmean")
    return packed, scale, codes


def prom_quantize_activation_absmax(x, eps: float = 1e-5, q=None, scale=None, stream=None):
    """x: float32 [n, ...] device.  Returns (int8 tensor of x's shape, scale float32 [n])."""
    import torch
    if not (x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() >= 1):
        raise TypeError("x must be a contiguous float32 device tensor [n, ...]")
    n = x.shape[0]
    per = x.numel() // n
    if q is None:
        q = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    if scale is None:
        scale = torch.empty(n, dtype=torch.float32, device=x.device)
    _check(load_library().prom_quantize_activation_absmax(x.data_ptr(), n, per, float(eps), q.data_ptr(),
                                                          scale.data_ptr(), _stream_ptr(stream)),
           "prom_quantize_activation_absmax")
    return q, scale


def prom_pw_conv_dynq(x, w_packed, cout: int, x_step, w_scale, bias=None, relu: bool = False,
                      eps: float = 1e-5, q=None, amax=None, scale=None, stream=None):
    """x: int8 [n,h,w,cin] device; x_step float32 [n], w_scale float32 [cout], bias float32 [cout]
    or None (device).  Returns (q int8 [n,h,w,cout], amax float32 [n], scale float32 [n])."""
    import torch
    _dev_i8(x, "x")
    n, h, w, cin = x.shape
    for name, t, cnt in (("x_step", x_step, n), ("w_scale", w_scale, cout), ("bias", bias, cout)):
        if t is None and name == "bias":
            continue
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == cnt):
            raise TypeError(f"{name} must be a contiguous float32 device tensor of {cnt} elements")
    if q is None:
        q = torch.empty((n, h, w, cout), dtype=torch.int8, device=x.device)
    _dev_i8(q, "q")
    if amax is None:
        amax = torch.empty(n, dtype=torch.float32, device=x.device)
    if scale is None:
        scale = torch.empty(n, dtype=torch.float32, device=x.device)
    _check(load_library().prom_pw_conv_dynq(
        x.data_ptr(), n, h, w, cin, w_packed.data_ptr(), int(cout), x_step.data_ptr(), w_scale.data_ptr(),
        bias.data_ptr() if bias is not None else None, int(bool(relu)), float(eps), q.data_ptr(),
        amax.data_ptr(), scale.data_ptr(), _stream_ptr(stream)), "prom_pw_conv_dynq")
    return q, amax, scale


def prom_quantize_dw_absmax(w, eps: float = 1e-5, stream=None):
    """w: float32 [c, 3, 3] device.  Returns (int8 [3, 3, c] device tensor, scale float32 [c])."""
    import torch
    if not (w.is_cuda and w.dtype == torch.float32 and w.is_contiguous() and tuple(w.shape[1:]) == (3, 3)):
        raise TypeError("w must be a contiguous float32 [c, 3, 3] device tensor")
    c = w.shape[0]
    wq = torch.empty((3, 3, c), dtype=torch.int8, device=w.device)
    scale = torch.empty(c, dtype=torch.float32, device=w.device)
    _check(load_library().prom_quantize_dw_absmax(w.data_ptr(), c, float(eps), wq.data_ptr(), scale.data_ptr(),
                                                  _stream_ptr(stream)), "prom_quantize_dw_absmax")
    return wq, scale


def prom_quantize_gconv_absmax(w, eps: float = 1e-5, stream=None):
    """w: float32 [c, group_size, 3, 3] device.  Returns (int8 [3, 3, c, group_size], scale float32 [c])."""
    import torch
    if not (w.is_cuda and w.dtype == torch.float32 and w.is_contiguous() and w.dim() == 4
            and tuple(w.shape[2:]) == (3, 3)):
        raise TypeError("w must be a contiguous float32 [c, group_size, 3, 3] device tensor")
    c, gs = int(w.shape[0]), int(w.shape[1])
    wq = torch.empty((3, 3, c, gs), dtype=torch.int8, device=w.device)
    scale = torch.empty(c, dtype=torch.float32, device=w.device)
    _check(load_library().prom_quantize_gconv_absmax(w.data_ptr(), c, gs, float(eps), wq.data_ptr(),
                                                     scale.data_ptr(), _stream_ptr(stream)),
           "prom_quantize_gconv_absmax")
    return wq, scale


def prom_block_is_fused(n: int, h: int, w: int, cin: int, chid: int, cout: int, stride: int) -> bool:
    rc = load_library().prom_block_is_fused(n, h, w, cin, chid, cout, stride)
    if rc < 0:
        raise PromError(rc, "prom_block_is_fused")
    return bool(rc)


def prom_pw_plan_query(n: int, h: int, w: int, cin: int, cout: int) -> dict:
    """Launch plan the library picks for a shape: tiles per wave, pixel tiles, workgroups per
    chunk and activation load width."""
    p = _PlanC()
    lb = ctypes.c_int(0)
    _check(load_library().prom_pw_plan_query(n, h, w, cin, cout, ctypes.byref(p), ctypes.byref(lb)),
           "prom_pw_plan_query")
    return {"tiles_per_wave": p.tiles_per_wave, "pixel_tiles": p.pixel_tiles,
            "workgroups": p.workgroups, "row_waves": p.row_waves, "k_outer": p.k_outer, "load_bytes": lb.value}


def prom_pw_batch_class(n: int, h: int, w: int, cin: int, cout: int) -> int:
    """0: launched alone, 1: joins the launch of small layers, 2: the launch of large layers."""
    rc = load_library().prom_pw_batch_class(n, h, w, cin, cout)
    if rc < 0:
        raise PromError(rc, "prom_pw_batch_class")
    return rc


def prom_pw_batchable(n: int, h: int, w: int, cin: int, cout: int) -> bool:
    rc = load_library().prom_pw_batchable(n, h, w, cin, cout)
    if rc < 0:
        raise PromError(rc, "prom_pw_batchable")
    return bool(rc)


class PwSequence:
    """A prebuilt array of prom_pw_layer_t; run() enqueues all layers with one C call.
    Keeps references to every tensor it points at."""

    def __init__(self, layers):
        """layers: iterable of (x, w_packed, cout, Requant, residual_or_None, y) device tensors."""
        layers = list(layers)
        self._keep = layers
        self._arr = (_PwLayerC * len(layers))()
        for i, (x, wp, cout, rq, res, y) in enumerate(layers):
            _dev_i8(x, "x")
            _dev_i8(y, "y")
            n, h, w, cin = x.shape
            c = self._arr[i]
            c.x, c.n, c.h, c.w, c.cin = x.data_ptr(), n, h, w, cin
            c.w_packed, c.cout, c.rq = wp.data_ptr(), int(cout), rq._c()
            c.residual = res.data_ptr() if res is not None else None
            c.y = y.data_ptr()
        self.count = len(layers)

    def run(self, stream=None):
        bad = ctypes.c_int(-1)
        rc = load_library().prom_pw_conv_sequence(self._arr, self.count, ctypes.byref(bad),
                                                  _stream_ptr(stream))
        if rc != PROM_OK:
            raise PromError(rc, f"prom_pw_conv_sequence (layer {bad.value})")


def prom_pw_conv_sequence(layers, stream=None):
    PwSequence(layers).run(stream)


class DwSequence:
    """A prebuilt array of prom_dw_layer_t; run() enqueues all layers with one C call.
    Keeps references to every tensor it points at."""

    def __init__(self, layers):
        """layers: iterable of (x, w_dw, stride, Requant, y) device tensors."""
        layers = list(layers)
        self._keep = layers
        self._arr = (_DwLayerC * len(layers))()
        for i, (x, w_dw, stride, rq, y) in enumerate(layers):
            _dev_i8(x, "x")
            _dev_i8(y, "y")
            _dev_i8(w_dw, "w_dw")
            n, h, w, c = x.shape
            l = self._arr[i]
            l.x, l.n, l.h, l.w, l.c = x.data_ptr(), n, h, w, c
            l.w_dw, l.stride, l.rq, l.y = w_dw.data_ptr(), int(stride), rq._c(), y.data_ptr()
        self.count = len(layers)

    def run(self, stream=None):
        bad = ctypes.c_int(-1)
        rc = load_library().prom_dw_conv_sequence(self._arr, self.count, ctypes.byref(bad), _stream_ptr(stream))
        if rc != PROM_OK:
            raise PromError(rc, f"prom_dw_conv_sequence (layer {bad.value})")


def prom_dw_conv_sequence(layers, stream=None):
    DwSequence(layers).run(stream)


class GconvSequence:
    """A prebuilt array of prom_gconv_layer_t; run() enqueues all layers with one C call.
    Keeps references to every tensor it points at."""

    def __init__(self, layers):
        """layers: iterable of (x, w_g, stride, Requant, y, w_frag or None) device tensors;
        w_g is [3][3][c][group_size]."""
        layers = list(layers)
        self._keep = layers
        self._arr = (_GconvLayerC * len(layers))()
        for i, (x, w_g, stride, rq, y, w_frag) in enumerate(layers):
            _dev_i8(x, "x")
            _dev_i8(y, "y")
            _dev_i8(w_g, "w_g")
            n, h, w, c = x.shape
            if w_g.dim() != 4 or tuple(w_g.shape[:3]) != (3, 3, c):
                raise ValueError("w_g must be [3][3][c][group_size]")
            l = self._arr[i]
            l.x, l.n, l.h, l.w, l.c = x.data_ptr(), n, h, w, c
            l.w_g, l.group_size, l.stride = w_g.data_ptr(), int(w_g.shape[3]), int(stride)
            l.w_frag = w_frag.data_ptr() if w_frag is not None else None
            l.rq, l.y = rq._c(), y.data_ptr()
        self.count = len(layers)

    def run(self, stream=None):
        bad = ctypes.c_int(-1)
        rc = load_library().prom_gconv3x3_sequence(self._arr, self.count, ctypes.byref(bad), _stream_ptr(stream))
        if rc != PROM_OK:
            raise PromError(rc, f"prom_gconv3x3_sequence (layer {bad.value})")


def prom_gconv3x3_sequence(layers, stream=None):
    GconvSequence(layers).run(stream)


def prom_copy_bytes(src, dst, nbytes: Optional[int] = None, stream=None):
    if nbytes is None:
        nbytes = src.numel() * src.element_size()
    _check(load_library().prom_copy_bytes(src.data_ptr(), dst.data_ptr(), int(nbytes),
                                          _stream_ptr(stream)), "prom_copy_bytes")
    return dst


def prom_stream_read(src, sink, nbytes: Optional[int] = None, stream=None):
    if nbytes is None:
        nbytes = src.numel() * src.element_size()
    _check(load_library().prom_stream_read(src.data_ptr(), int(nbytes), sink.data_ptr(), _stream_ptr(stream)),
           "prom_stream_read")


def prom_stream_write(dst, value: int = 0, nbytes: Optional[int] = None, stream=None):
    if nbytes is None:
        nbytes = dst.numel() * dst.element_size()
    _check(load_library().prom_stream_write(dst.data_ptr(), int(nbytes), int(value), _stream_ptr(stream)),
           "prom_stream_write")


def prom_mfma_i8_loop(iters: int, sink, stream=None) -> int:
    """Launches the register-resident int8 MFMA loop; returns the operations it performs."""
    ops = int(load_library().prom_mfma_i8_loop(int(iters), sink.data_ptr(), _stream_ptr(stream)))
    if ops < 0:
        raise PromError(ops, "prom_mfma_i8_loop")
    return ops


def prom_requant_check(rq: Requant, cin: int) -> int:
    """Opt-in check of the requantisation preconditions (copies the arrays to the host).  Returns -1
    if they hold, else the first offending channel."""
    rqc = rq._c()
    bad = ctypes.c_int(-1)
    rc = load_library().prom_requant_check(ctypes.byref(rqc), int(rq.bias.numel()), int(cin), ctypes.byref(bad))
    if rc == PROM_OK:
        return -1
    if rc == -1 and bad.value >= 0:
        return bad.value
    raise PromError(rc, "prom_requant_check")
