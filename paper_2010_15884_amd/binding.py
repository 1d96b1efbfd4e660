"""ctypes binding of libsysconv.so: argument marshalling only.

Every function has the name and the arguments of the C entry point it calls
(see include/sysconv.h); tensors are torch CUDA tensors used purely as device
memory, and the stream is torch's current stream unless one is given.  There is
no fallback: if the library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsysconv.so")

SYS_OK, SYS_ERR_NULL, SYS_ERR_SIZE, SYS_ERR_ALIAS, SYS_ERR_UNSUPPORTED, SYS_ERR_HIP = range(6)
(SYS_PROJ_AUTO, SYS_PROJ_FBS, SYS_PROJ_BFS, SYS_PROJ_SBM, SYS_PROJ_BSM, SYS_PROJ_FSM, SYS_PROJ_FFS,
 SYS_PROJ_MFMA) = range(8)
PROJECTIONS = {"AUTO": SYS_PROJ_AUTO, "FBS": SYS_PROJ_FBS, "BFS": SYS_PROJ_BFS, "SBM": SYS_PROJ_SBM,
               "BSM": SYS_PROJ_BSM, "FSM": SYS_PROJ_FSM, "FFS": SYS_PROJ_FFS, "MFMA": SYS_PROJ_MFMA}
SYS_ERR_DESIGN = 6
SYS_MAX_K1D = 64
SYS_MAX_K2D = 15

EXPORTS = ["sys_conv1d", "sys_conv1d_strided", "sys_conv2d", "sys_conv1d_has", "sys_conv1d_strided_has",
           "sys_conv2d_has", "sys_conv2d_strided", "sys_conv2d_strided_has", "sys_stt_check", "sys_conv1d_stt", "sys_copy_f32", "sys_alu_yardstick_f32", "sys_status_string",
           "sys_projection_name", "sys_last_hip_error", "sys_version"]

_lib = None


class SttDesign(ctypes.Structure):
    """sys_stt_design_t: transform rows P and s over (c, q) and the dependence vectors of X, W, Z."""
    _fields_ = [("alloc", ctypes.c_int * 2), ("sched", ctypes.c_int * 2),
                ("x_passed", ctypes.c_int), ("dep_x", ctypes.c_int * 2),
                ("w_passed", ctypes.c_int), ("dep_w", ctypes.c_int * 2),
                ("dep_z", ctypes.c_int * 2)]


def stt_design(alloc, sched, dep_x=None, dep_w=None, dep_z=(0, 1)) -> SttDesign:
    """Build a design; ``dep_x`` / ``dep_w`` = None means the variable is loaded by every PE."""
    d = SttDesign()
    d.alloc[:] = [int(v) for v in alloc]
    d.sched[:] = [int(v) for v in sched]
    d.x_passed = int(dep_x is not None)
    d.dep_x[:] = [int(v) for v in (dep_x or (0, 0))]
    d.w_passed = int(dep_w is not None)
    d.dep_w[:] = [int(v) for v in (dep_w or (0, 0))]
    d.dep_z[:] = [int(v) for v in dep_z]
    return d


def named_design(name: str) -> SttDesign:
    """One of the paper's six designs (Section 3.1, Table 2) as a sys_stt_design_t."""
    from . import schedule_model as sm
    t, e = sm.TRANSFORMS[name], sm.DEPENDENCES[name]
    return stt_design(t.alloc, t.sched, e.get("X"), e.get("W"), e["Z"])


class SysconvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"sysconv status {status}: {message}")
        self.status = status


def lib() -> ctypes.CDLL:
    """Load libsysconv.so (built by ``python -m paper_2010_15884_amd.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2010_15884_amd.build` "
                "(there is no fallback path)")
        # The tensors and streams handed to the library come from torch, so both must
        # talk to ONE HIP runtime.  torch ships its own libamdhip64 under the same soname
        # as the system's; whichever is loaded first serves the whole process, so torch
        # has to come first.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, fp, sz, ci = ctypes.c_void_p, ctypes.POINTER(ctypes.c_float), ctypes.c_size_t, ctypes.c_int
        L.sys_conv1d.argtypes = [vp, sz, fp, ci, vp, ci, vp]
        L.sys_conv1d.restype = ci
        L.sys_conv2d.argtypes = [vp, ci, ci, sz, fp, ci, ci, vp, sz, ci, vp]
        L.sys_conv2d.restype = ci
        L.sys_conv1d_strided.argtypes = [vp, sz, fp, ci, ci, vp, ci, vp]
        L.sys_conv1d_strided.restype = ci
        L.sys_conv1d_strided_has.argtypes = [ci, ci, ci]
        L.sys_conv1d_strided_has.restype = ci
        L.sys_stt_check.argtypes = [ctypes.POINTER(SttDesign), ci]
        L.sys_stt_check.restype = ci
        L.sys_conv1d_stt.argtypes = [vp, sz, fp, ci, vp, ctypes.POINTER(SttDesign), vp]
        L.sys_conv1d_stt.restype = ci
        L.sys_conv2d_strided.argtypes = [vp, ci, ci, sz, fp, ci, ci, ci, vp, sz, ci, vp]
        L.sys_conv2d_strided.restype = ci
        L.sys_conv2d_strided_has.argtypes = [ci, ci, ci, ci]
        L.sys_conv2d_strided_has.restype = ci
        L.sys_conv1d_has.argtypes = [ci, ci]
        L.sys_conv1d_has.restype = ci
        L.sys_conv2d_has.argtypes = [ci, ci, ci]
        L.sys_conv2d_has.restype = ci
        L.sys_copy_f32.argtypes = [vp, vp, sz, vp]
        L.sys_copy_f32.restype = ci
        L.sys_alu_yardstick_f32.argtypes = [vp, ci, ci, vp]
        L.sys_alu_yardstick_f32.restype = ctypes.c_longlong
        L.sys_status_string.argtypes = [ci]
        L.sys_status_string.restype = ctypes.c_char_p
        L.sys_projection_name.argtypes = [ci]
        L.sys_projection_name.restype = ctypes.c_char_p
        L.sys_last_hip_error.argtypes = []
        L.sys_last_hip_error.restype = ci
        L.sys_version.argtypes = []
        L.sys_version.restype = ci
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().sys_status_string(int(status)).decode()


def projection_name(projection: int) -> str:
    return lib().sys_projection_name(int(projection)).decode()


def _check(status: int) -> None:
    if status != SYS_OK:
        msg = status_string(status)
        if status == SYS_ERR_HIP:
            msg += f" [hipError {lib().sys_last_hip_error()}]"
        raise SysconvError(status, msg)


def _proj(projection) -> int:
    if isinstance(projection, str):
        return PROJECTIONS[projection.upper()]
    return int(projection)


def _taps(w) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(w, dtype=np.float32))


def _stream_handle(stream) -> Optional[int]:
    """The hipStream_t to launch on: the caller's, else torch's current stream."""
    if stream is not None:
        return int(stream)
    import torch
    raw = getattr(torch._C, "_cuda_getCurrentRawStream", None)      # the short way, when this torch has it
    if raw is not None:
        return raw(torch.cuda.current_device())
    return torch.cuda.current_stream().cuda_stream


def _device_f32(t, what):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.float32:
        raise TypeError(f"{what} must be a float32 CUDA tensor")
    return t


def _room_1d(d_y, m):
    """The library writes m floats through the pointer it is given: make sure the tensor has them."""
    _device_f32(d_y, "d_y")
    if d_y.dim() != 1 or not d_y.is_contiguous() or d_y.numel() < m:
        raise ValueError(f"d_y must be a contiguous 1-D tensor with room for {m} outputs")


def sys_conv1d(d_x, h_w, d_y=None, projection="AUTO", stream=None):
    """y[c] = sum_q x[c+q] w[q].  d_x: 1-D float32 CUDA tensor; h_w: host taps.
    Returns d_y (allocated with torch if not given)."""
    import torch
    _device_f32(d_x, "d_x")
    if d_x.dim() != 1 or not d_x.is_contiguous():
        raise ValueError("d_x must be a contiguous 1-D tensor")
    w = _taps(h_w)
    n, k = d_x.shape[0], w.shape[0]
    if d_y is None:
        d_y = torch.empty(max(n - k + 1, 0), dtype=torch.float32, device=d_x.device)
    _room_1d(d_y, max(n - k + 1, 0))
    _check(lib().sys_conv1d(d_x.data_ptr(), n, w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), k,
                            d_y.data_ptr(), _proj(projection), _stream_handle(stream)))
    return d_y


def sys_conv1d_strided(d_x, h_w, stride, d_y=None, projection="AUTO", stream=None):
    """y[c] = sum_q x[stride*c+q] w[q], (n-k)//stride + 1 outputs.  Arguments as sys_conv1d."""
    import torch
    _device_f32(d_x, "d_x")
    if d_x.dim() != 1 or not d_x.is_contiguous():
        raise ValueError("d_x must be a contiguous 1-D tensor")
    w = _taps(h_w)
    n, k, stride = d_x.shape[0], w.shape[0], int(stride)
    m = (n - k) // stride + 1 if (stride >= 1 and n >= k) else 0
    if d_y is None:
        d_y = torch.empty(m, dtype=torch.float32, device=d_x.device)
    _room_1d(d_y, m)
    _check(lib().sys_conv1d_strided(d_x.data_ptr(), n, w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), k, stride,
                                    d_y.data_ptr(), _proj(projection), _stream_handle(stream)))
    return d_y


def sys_stt_check(design: SttDesign, k: int) -> int:
    """Status the library gives this design for a k-tap filter (SYS_OK, SYS_ERR_DESIGN, ...)."""
    return int(lib().sys_stt_check(ctypes.byref(design), int(k)))


def sys_conv1d_stt(d_x, h_w, design: SttDesign, d_y=None, stream=None):
    """sys_conv1d computed by the generic space-time-transform kernel for ``design``."""
    import torch
    _device_f32(d_x, "d_x")
    if d_x.dim() != 1 or not d_x.is_contiguous():
        raise ValueError("d_x must be a contiguous 1-D tensor")
    w = _taps(h_w)
    n, k = d_x.shape[0], w.shape[0]
    if d_y is None:
        d_y = torch.empty(max(n - k + 1, 0), dtype=torch.float32, device=d_x.device)
    _room_1d(d_y, max(n - k + 1, 0))
    _check(lib().sys_conv1d_stt(d_x.data_ptr(), n, w.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), k,
                                d_y.data_ptr(), ctypes.byref(design), _stream_handle(stream)))
    return d_y


def sys_conv2d(d_x, h_f, d_y=None, projection="AUTO", stream=None):
    """y[r][c] = sum_p sum_q x[r+p][c+q] f[p][q].  d_x: 2-D float32 CUDA tensor whose
    rows are contiguous (stride(1) == 1; stride(0) is the pitch); h_f: host kh x kw taps."""
    import torch
    _device_f32(d_x, "d_x")
    if d_x.dim() != 2 or d_x.stride(1) != 1:
        raise ValueError("d_x must be 2-D with unit column stride")
    f = _taps(h_f)
    if f.ndim != 2:
        raise ValueError("h_f must be 2-D")
    h, w = d_x.shape
    kh, kw = f.shape
    if d_y is None:
        d_y = torch.empty((max(h - kh + 1, 0), max(w - kw + 1, 0)), dtype=torch.float32, device=d_x.device)
    _device_f32(d_y, "d_y")
    if d_y.dim() != 2 or d_y.stride(1) != 1:
        raise ValueError("d_y must be 2-D with unit column stride")
    if d_y.shape[0] < max(h - kh + 1, 0) or d_y.shape[1] < max(w - kw + 1, 0):
        raise ValueError(f"d_y must have room for {h - kh + 1} x {w - kw + 1} outputs")
    _check(lib().sys_conv2d(d_x.data_ptr(), h, w, d_x.stride(0),
                            f.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), kh, kw,
                            d_y.data_ptr(), d_y.stride(0), _proj(projection), _stream_handle(stream)))
    return d_y


def sys_conv2d_strided(d_x, h_f, stride, d_y=None, projection="AUTO", stream=None):
    """y[r][c] = sum_p sum_q x[stride*r+p][stride*c+q] f[p][q].  Arguments as sys_conv2d."""
    import torch
    _device_f32(d_x, "d_x")
    if d_x.dim() != 2 or d_x.stride(1) != 1:
        raise ValueError("d_x must be 2-D with unit column stride")
    f = _taps(h_f)
    if f.ndim != 2:
        raise ValueError("h_f must be 2-D")
    h, w = d_x.shape
    kh, kw = f.shape
    stride = int(stride)
    ok = stride >= 1 and h >= kh and w >= kw
    oh, ow = ((h - kh) // stride + 1, (w - kw) // stride + 1) if ok else (0, 0)
    if d_y is None:
        d_y = torch.empty((oh, ow), dtype=torch.float32, device=d_x.device)
    _device_f32(d_y, "d_y")
    if d_y.dim() != 2 or d_y.stride(1) != 1:
        raise ValueError("d_y must be 2-D with unit column stride")
    if d_y.shape[0] < oh or d_y.shape[1] < ow:
        raise ValueError(f"d_y must have room for {oh} x {ow} outputs")
    _check(lib().sys_conv2d_strided(d_x.data_ptr(), h, w, d_x.stride(0),
                                    f.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), kh, kw, stride,
                                    d_y.data_ptr(), d_y.stride(0), _proj(projection), _stream_handle(stream)))
    return d_y


def sys_conv2d_strided_has(projection, kh: int, kw: int, stride: int) -> bool:
    return bool(lib().sys_conv2d_strided_has(_proj(projection), int(kh), int(kw), int(stride)))


def sys_conv1d_has(projection, k: int) -> bool:
    return bool(lib().sys_conv1d_has(_proj(projection), int(k)))


def sys_conv1d_strided_has(projection, k: int, stride: int) -> bool:
    return bool(lib().sys_conv1d_strided_has(_proj(projection), int(k), int(stride)))


def sys_conv2d_has(projection, kh: int, kw: int) -> bool:
    return bool(lib().sys_conv2d_has(_proj(projection), int(kh), int(kw)))


def sys_copy_f32(d_src, d_dst, stream=None):
    _device_f32(d_src, "d_src")
    _device_f32(d_dst, "d_dst")
    if d_src.numel() != d_dst.numel() or not d_src.is_contiguous() or not d_dst.is_contiguous():
        raise ValueError("copy needs two contiguous tensors of equal size")
    _check(lib().sys_copy_f32(d_src.data_ptr(), d_dst.data_ptr(), d_src.numel(), _stream_handle(stream)))
    return d_dst


def sys_alu_yardstick_f32(d_out, workgroups: int, trips: int, stream=None) -> int:
    """Enqueue the register-only multiply-add loop; returns the number of multiply-adds it performs."""
    _device_f32(d_out, "d_out")
    if not d_out.is_contiguous() or d_out.numel() < int(workgroups) * 256:
        raise ValueError("d_out must be contiguous with room for workgroups * 256 floats")
    n = int(lib().sys_alu_yardstick_f32(d_out.data_ptr(), int(workgroups), int(trips), _stream_handle(stream)))
    if n < 0:
        _check(-n)
    return n


def sys_version() -> int:
    return int(lib().sys_version())
