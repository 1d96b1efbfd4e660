"""CPU oracle for 1-D / 2-D valid convolution -- TEST INFRASTRUCTURE ONLY.

A thin numpy/ctypes wrapper over ``conv_oracle.c`` (plain C, fp64 sums), which
writes out the paper's Eq. 2 (Section 3.1) and Eq. 3 (Section 5) as loops.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The GPU library never does, and this
package never imports the GPU library.

Pins (see ``tests/test_oracle_pins.py`` and ``tests/test_ure_recurrences.py``):
hand-expanded sums, delta filters, linearity, separability, constant / ramp /
box closed forms, integer-exact data, numpy's and torch's float64 routines as a
library special case, the paper's recurrence equations (Section 3.1, Table 2,
Section 5) evaluated literally, and the printed values of Table 4; the strided
forms also against hand sums, every stride-th output of the stride-1 forms, numpy's
correlate resp. torch's conv2d(stride=2) in float64, delta filters, and (1-D) the
stride-2 recurrences of Table 2.  The scale routines (``absdot*``) are pinned by hand-expanded
sums with distinct magnitudes (``tests/golden/hand_sums.txt``) and, bit for bit, by the pinned
convolutions applied to the magnitudes; the pitch arguments of the C routines by padded buffers
whose padding holds NaN resp. a sentinel.
Nothing here is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "libconv_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile conv_oracle.c with gcc (no fast-math: summation order is kept)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        for name in ("oracle_conv1d", "oracle_absdot1d"):
            fn = getattr(lib, name)
            fn.argtypes = [fp, ctypes.c_size_t, fp, ctypes.c_int, dp, ctypes.c_int]
            fn.restype = ctypes.c_int
        for name in ("oracle_conv1d_strided", "oracle_absdot1d_strided"):
            fn = getattr(lib, name)
            fn.argtypes = [fp, ctypes.c_size_t, fp, ctypes.c_int, ctypes.c_int, dp, ctypes.c_int]
            fn.restype = ctypes.c_int
        for name in ("oracle_conv2d", "oracle_absdot2d"):
            fn = getattr(lib, name)
            fn.argtypes = [fp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t,
                           fp, ctypes.c_int, ctypes.c_int,
                           dp, ctypes.c_size_t, ctypes.c_int]
            fn.restype = ctypes.c_int
        for name in ("oracle_conv2d_strided", "oracle_absdot2d_strided"):
            fn = getattr(lib, name)
            fn.argtypes = [fp, ctypes.c_int, ctypes.c_int, ctypes.c_size_t,
                           fp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                           dp, ctypes.c_size_t, ctypes.c_int]
            fn.restype = ctypes.c_int
        lib.oracle_threads.argtypes = [ctypes.c_int]
        lib.oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f32(a, ndim):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.ndim != ndim:
        raise ValueError(f"expected {ndim}-D array, got shape {a.shape}")
    return a


def _fptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def threads_used(nthreads: int) -> int:
    return int(_load().oracle_threads(int(nthreads)))


def _run1d(fname, x, w, nthreads):
    x = _f32(x, 1)
    w = _f32(w, 1)
    n, k = x.shape[0], w.shape[0]
    if k < 1 or k > n:
        raise ValueError("need 1 <= k <= n")
    y = np.empty(n - k + 1, dtype=np.float64)
    rc = getattr(_load(), fname)(_fptr(x), n, _fptr(w), k, _dptr(y), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"{fname} failed with status {rc}")
    return y


def _run1d_strided(fname, x, w, stride, nthreads):
    x = _f32(x, 1)
    w = _f32(w, 1)
    n, k = x.shape[0], w.shape[0]
    if k < 1 or k > n or stride < 1:
        raise ValueError("need 1 <= k <= n and stride >= 1")
    y = np.empty((n - k) // stride + 1, dtype=np.float64)
    rc = getattr(_load(), fname)(_fptr(x), n, _fptr(w), k, int(stride), _dptr(y), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"{fname} failed with status {rc}")
    return y


_SENTINEL = -12345.678        # what the gaps between result rows hold before the call


def _padded_input(x, x_pitch):
    """The image laid out with a row stride of x_pitch elements; the padding holds NaN so that a
    read outside the image shows up in the result."""
    h, w_img = x.shape
    if x_pitch is None or x_pitch == w_img:
        return x, w_img
    if x_pitch < w_img:
        raise ValueError("x_pitch must be >= the image width")
    buf = np.full((h, x_pitch), np.nan, dtype=np.float32)
    buf[:, :w_img] = x
    return buf, x_pitch


def _pitched_output(shape, y_pitch):
    """Result buffer with a row stride of y_pitch elements, padding pre-set to a sentinel that a
    correct oracle leaves alone."""
    oh, ow = shape
    if y_pitch is None or y_pitch == ow:
        return np.empty((oh, ow), dtype=np.float64), ow
    if y_pitch < ow:
        raise ValueError("y_pitch must be >= the output width")
    return np.full((oh, y_pitch), _SENTINEL, dtype=np.float64), y_pitch


def _unpad_output(buf, shape):
    oh, ow = shape
    if buf.shape[1] != ow and not np.all(buf[:, ow:] == _SENTINEL):
        raise RuntimeError("the oracle wrote between the rows of its result")
    return np.ascontiguousarray(buf[:, :ow])



def _run2d(fname, x, f, nthreads, x_pitch=None, y_pitch=None):
    x = _f32(x, 2)
    f = _f32(f, 2)
    h, w_img = x.shape
    kh, kw = f.shape
    if kh < 1 or kw < 1 or kh > h or kw > w_img:
        raise ValueError("filter must fit inside the image")
    shape = (h - kh + 1, w_img - kw + 1)
    xin, xp = _padded_input(x, x_pitch)
    y, yp = _pitched_output(shape, y_pitch)
    rc = getattr(_load(), fname)(_fptr(xin), h, w_img, xp, _fptr(f), kh, kw, _dptr(y), yp, int(nthreads))
    if rc != 0:
        raise RuntimeError(f"{fname} failed with status {rc}")
    return _unpad_output(y, shape)


def _run2d_strided(fname, x, f, stride, nthreads, x_pitch=None, y_pitch=None):
    x = _f32(x, 2)
    f = _f32(f, 2)
    h, w_img = x.shape
    kh, kw = f.shape
    if kh < 1 or kw < 1 or kh > h or kw > w_img or stride < 1:
        raise ValueError("filter must fit inside the image and stride must be >= 1")
    shape = ((h - kh) // stride + 1, (w_img - kw) // stride + 1)
    xin, xp = _padded_input(x, x_pitch)
    y, yp = _pitched_output(shape, y_pitch)
    rc = getattr(_load(), fname)(_fptr(xin), h, w_img, xp, _fptr(f), kh, kw, int(stride), _dptr(y), yp,
                                 int(nthreads))
    if rc != 0:
        raise RuntimeError(f"{fname} failed with status {rc}")
    return _unpad_output(y, shape)


def conv1d(x, w, nthreads: int = 1) -> np.ndarray:
    """Eq. 2: y[c] = sum_q x[c+q] * w[q]; fp32 inputs, fp64 result, length n-k+1."""
    return _run1d("oracle_conv1d", x, w, nthreads)


def conv1d_strided(x, w, stride: int, nthreads: int = 1) -> np.ndarray:
    """Table 2, row 3 right, read as y[c] = sum_q x[stride*c+q] * w[q]; length (n-k)//stride + 1."""
    return _run1d_strided("oracle_conv1d_strided", x, w, stride, nthreads)


def absdot1d_strided(x, w, stride: int, nthreads: int = 1) -> np.ndarray:
    return _run1d_strided("oracle_absdot1d_strided", x, w, stride, nthreads)


def conv2d(x, f, nthreads: int = 1, x_pitch=None, y_pitch=None) -> np.ndarray:
    """Eq. 3 on a row-major image: y[r][c] = sum_p sum_q f[p][q] * x[r+p][c+q].

    x_pitch / y_pitch (elements) make the C routine work on buffers whose rows are further apart
    than the image resp. the result is wide; the returned array is always the compact result."""
    return _run2d("oracle_conv2d", x, f, nthreads, x_pitch, y_pitch)


def conv2d_strided(x, f, stride: int, nthreads: int = 1, x_pitch=None, y_pitch=None) -> np.ndarray:
    """y[r][c] = sum_p sum_q f[p][q] * x[stride*r+p][stride*c+q] (the same stride on both axes)."""
    return _run2d_strided("oracle_conv2d_strided", x, f, stride, nthreads, x_pitch, y_pitch)


def absdot2d_strided(x, f, stride: int, nthreads: int = 1, x_pitch=None, y_pitch=None) -> np.ndarray:
    return _run2d_strided("oracle_absdot2d_strided", x, f, stride, nthreads, x_pitch, y_pitch)


def absdot1d(x, w, nthreads: int = 1) -> np.ndarray:
    """sum_q |x[c+q]| |w[q]| -- the scale of the parity metric."""
    return _run1d("oracle_absdot1d", x, w, nthreads)


def absdot2d(x, f, nthreads: int = 1, x_pitch=None, y_pitch=None) -> np.ndarray:
    """sum_p sum_q |x[r+p][c+q]| |f[p][q]| -- the scale of the 2-D parity metric."""
    return _run2d("oracle_absdot2d", x, f, nthreads, x_pitch, y_pitch)


def max_rel_err(y_test, y_ref, scale) -> float:
    """max_i |y_test[i] - y_ref[i]| / scale[i]   (all compared in fp64).

    Where scale[i] == 0 every term of the sum is zero, so the only acceptable
    difference is exactly 0; anything else is reported as infinity.
    """
    y_test = np.asarray(y_test, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    scale = np.asarray(scale, dtype=np.float64)
    if y_test.shape != y_ref.shape or y_ref.shape != scale.shape:
        raise ValueError(f"shape mismatch {y_test.shape} {y_ref.shape} {scale.shape}")
    if y_test.size == 0:
        return 0.0
    diff = np.abs(y_test - y_ref)
    if not np.all(np.isfinite(y_test)):
        return float("inf")
    zero = scale == 0
    if np.any(diff[zero] != 0):
        return float("inf")
    safe = np.where(zero, 1.0, scale)
    return float(np.max(np.where(zero, 0.0, diff / safe)))
