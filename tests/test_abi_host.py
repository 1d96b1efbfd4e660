"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2010_15884_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FP = ctypes.POINTER(ctypes.c_float)


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sysconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sys_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n


def test_strings_and_version():
    assert B.sys_version() >= 100
    assert B.status_string(B.SYS_OK) == "ok"
    for s in range(1, 6):
        assert B.status_string(s) not in ("ok", "unknown status")
    assert B.status_string(99) == "unknown status"
    assert [B.projection_name(p) for p in range(8)] == ["AUTO", "FBS", "BFS", "SBM", "BSM", "FSM", "FFS", "MFMA"]
    assert B.projection_name(17) == "?"


def _w(k):
    w = np.ones(max(k, 1), np.float32)
    return w, w.ctypes.data_as(FP)


# fake, 4-byte aligned, non-overlapping "device" addresses: validation never dereferences them
X, Y = 0x10000000, 0x40000000


@pytest.mark.parametrize("args,want", [
    ((None, 100, "w", 5, Y, 1), B.SYS_ERR_NULL),
    ((X, 100, None, 5, Y, 1), B.SYS_ERR_NULL),
    ((X, 100, "w", 5, None, 1), B.SYS_ERR_NULL),
    ((X, 100, "w", 0, Y, 1), B.SYS_ERR_SIZE),
    ((X, 100, "w", -3, Y, 1), B.SYS_ERR_SIZE),
    ((X, 4, "w", 5, Y, 1), B.SYS_ERR_SIZE),
    ((X, 0, "w", 1, Y, 1), B.SYS_ERR_SIZE),
    ((X, 100, "w", 65, Y, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, "w", 5, Y, 7), B.SYS_ERR_UNSUPPORTED),                     # MFMA is a 2-D projection
    ((X, 100, "w", 5, Y, 8), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, "w", 5, Y, -1), B.SYS_ERR_UNSUPPORTED),
    ((X + 2, 100, "w", 5, Y, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, "w", 5, X, 1), B.SYS_ERR_ALIAS),
    ((X, 100, "w", 5, X + 4 * 99, 1), B.SYS_ERR_ALIAS),
    ((X + 4 * 95, 100, "w", 5, X, 1), B.SYS_ERR_ALIAS),
])
def test_conv1d_validation(args, want):
    x, n, w, k, y, proj = args
    keep, wp = _w(k)
    got = B.lib().sys_conv1d(x, n, wp if w else None, k, y, proj, None)
    assert got == want, B.status_string(got)


@pytest.mark.parametrize("args,want", [
    ((None, 10, 10, 10, "f", 3, 3, Y, 8, 1), B.SYS_ERR_NULL),
    ((X, 10, 10, 10, None, 3, 3, Y, 8, 1), B.SYS_ERR_NULL),
    ((X, 10, 10, 10, "f", 3, 3, None, 8, 1), B.SYS_ERR_NULL),
    ((X, 10, 10, 10, "f", 0, 3, Y, 8, 1), B.SYS_ERR_SIZE),
    ((X, 10, 10, 10, "f", 11, 3, Y, 8, 1), B.SYS_ERR_SIZE),
    ((X, 10, 10, 10, "f", 3, 11, Y, 8, 1), B.SYS_ERR_SIZE),
    ((X, 10, 10, 9, "f", 3, 3, Y, 8, 1), B.SYS_ERR_SIZE),
    ((X, 10, 10, 10, "f", 3, 3, Y, 7, 1), B.SYS_ERR_SIZE),
    ((X, 0, 10, 10, "f", 1, 1, Y, 10, 1), B.SYS_ERR_SIZE),
    ((X, 100, 100, 100, "f", 16, 3, Y, 98, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, 100, 100, "f", 3, 16, Y, 98, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, 100, 100, "f", 3, 3, Y, 98, 9), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, 100, 100, "f", 3, 3, Y, 98, B.SYS_PROJ_BSM), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, 100, 100, "f", 4, 3, Y, 98, B.SYS_PROJ_BFS), B.SYS_ERR_UNSUPPORTED),
    ((X + 1, 100, 100, 100, "f", 3, 3, Y, 98, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, 100, 100, "f", 3, 3, X + 4 * 5000, 98, 1), B.SYS_ERR_ALIAS),
    ((X, 100, 100, 100, "f", 14, 3, Y, 98, B.SYS_PROJ_MFMA), B.SYS_ERR_UNSUPPORTED),    # MFMA: up to 13 x 13
    ((X, 100, 100, 100, "f", 3, 14, Y, 87, B.SYS_PROJ_MFMA), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, 100, 100, "f", 3, 3, X + 4 * 5000, 98, B.SYS_PROJ_MFMA), B.SYS_ERR_ALIAS),
    # rows longer than INT_MAX - 2048 would overflow the kernels' strip arithmetic
    ((X, 1, 2 ** 31 - 2047, 2 ** 31 - 2047, "f", 1, 3, 0x7000000000, 2 ** 31 - 2049, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 1, 2 ** 31 - 1, 2 ** 31 - 1, "f", 1, 1, 0x7000000000, 2 ** 31 - 1, 0), B.SYS_ERR_UNSUPPORTED),
])
def test_conv2d_validation(args, want):
    x, h, w, xp, f, kh, kw, y, yp, proj = args
    keep = np.ones(256, np.float32)
    got = B.lib().sys_conv2d(x, h, w, xp, keep.ctypes.data_as(FP) if f else None, kh, kw, y, yp, proj, None)
    assert got == want, B.status_string(got)


@pytest.mark.parametrize("amax,want", [(1e-33, B.SYS_ERR_UNSUPPORTED), (3e33, B.SYS_ERR_UNSUPPORTED),
                                        (float("inf"), B.SYS_ERR_ALIAS), (0.0, B.SYS_ERR_ALIAS),
                                        (1e-29, B.SYS_ERR_ALIAS), (1e29, B.SYS_ERR_ALIAS)])
def test_mfma_tap_range_is_checked_before_any_launch(amax, want):
    # The matrix-core path scales the taps by a power of two derived from the largest finite |f|, which has to lie
    # in [1e-30, 1e30] (or be 0).  The check comes last, so filters that pass it run into the planted aliasing.
    f = np.full(25, 0.0, np.float32)
    f[7] = amax
    f[3] = -amax / 2 if np.isfinite(amax) else 1.0
    if not np.isfinite(amax):
        f[7], f[3] = np.inf, 1e-33                 # a non-finite tap does not count; the largest finite one decides
        want = B.SYS_ERR_UNSUPPORTED
    got = B.lib().sys_conv2d(X, 100, 100, 100, f.ctypes.data_as(FP), 5, 5, X + 4 * 5000, 96, B.SYS_PROJ_MFMA, None)
    assert got == want, B.status_string(got)


def test_copy_validation():
    L = B.lib()
    assert L.sys_copy_f32(None, Y, 10, None) == B.SYS_ERR_NULL
    assert L.sys_copy_f32(X, None, 10, None) == B.SYS_ERR_NULL
    assert L.sys_copy_f32(X, Y, 0, None) == B.SYS_ERR_SIZE
    assert L.sys_copy_f32(X, X + 8, 10, None) == B.SYS_ERR_ALIAS
    assert L.sys_copy_f32(X + 1, Y, 10, None) == B.SYS_ERR_UNSUPPORTED


def test_alu_yardstick_validation():
    L = B.lib()
    assert L.sys_alu_yardstick_f32(None, 8, 8, None) == -B.SYS_ERR_NULL
    assert L.sys_alu_yardstick_f32(Y, 0, 8, None) == -B.SYS_ERR_SIZE
    assert L.sys_alu_yardstick_f32(Y, 8, 0, None) == -B.SYS_ERR_SIZE
    assert L.sys_alu_yardstick_f32(Y, (1 << 20) + 1, 8, None) == -B.SYS_ERR_SIZE
    assert L.sys_alu_yardstick_f32(Y + 2, 8, 8, None) == -B.SYS_ERR_UNSUPPORTED


def test_conv2d_has():
    assert B.sys_conv2d_has("FBS", 15, 15) and B.sys_conv2d_has("AUTO", 1, 9)
    assert not B.sys_conv2d_has("FBS", 16, 3)
    assert B.sys_conv2d_has("BFS", 3, 3) and B.sys_conv2d_has("BFS", 5, 5) and B.sys_conv2d_has("BFS", 11, 11)
    assert not B.sys_conv2d_has("BFS", 4, 5) and not B.sys_conv2d_has("SBM", 12, 12)
    assert not B.sys_conv2d_has(42, 3, 3)
    assert B.sys_conv2d_has("MFMA", 1, 1) and B.sys_conv2d_has("MFMA", 13, 13) and B.sys_conv2d_has("MFMA", 2, 13)
    assert not B.sys_conv2d_has("MFMA", 14, 3) and not B.sys_conv2d_has("MFMA", 3, 14)


def test_binding_rejects_host_tensors():
    torch = pytest.importorskip("torch")
    with pytest.raises(TypeError):
        B.sys_conv1d(torch.zeros(10), np.ones(3, np.float32))


@pytest.mark.parametrize("args,want", [
    ((None, 100, "w", 5, 2, Y, 1), B.SYS_ERR_NULL),
    ((X, 100, "w", 5, 2, None, 0), B.SYS_ERR_NULL),
    ((X, 100, "w", 5, 0, Y, 1), B.SYS_ERR_SIZE),
    ((X, 100, "w", 5, -2, Y, 1), B.SYS_ERR_SIZE),
    ((X, 4, "w", 5, 2, Y, 1), B.SYS_ERR_SIZE),
    ((X, 100, "w", 0, 2, Y, 1), B.SYS_ERR_SIZE),
    ((X, 100, "w", 65, 2, Y, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, "w", 5, 3, Y, 1), B.SYS_ERR_UNSUPPORTED),                  # only strides 1 and 2 are built
    ((X, 100, "w", 5, 2, Y, B.SYS_PROJ_SBM), B.SYS_ERR_UNSUPPORTED),     # stride 2 is an FBS design only
    ((X, 100, "w", 5, 2, Y, B.SYS_PROJ_BFS), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, "w", 5, 2, Y, 9), B.SYS_ERR_UNSUPPORTED),
    ((X + 2, 100, "w", 5, 2, Y, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, "w", 5, 2, X + 4 * 99, 0), B.SYS_ERR_ALIAS),
    ((X + 4 * 47, 100, "w", 5, 2, X, 0), B.SYS_ERR_ALIAS),               # 48 outputs: y = [X, X+192) touches x
    ((X, 100, "w", 5, 1, X, 1), B.SYS_ERR_ALIAS),                        # stride 1 goes through sys_conv1d's checks
    ((X, 100, "w", 65, 1, Y, 1), B.SYS_ERR_UNSUPPORTED),
])
def test_conv1d_strided_validation(args, want):
    x, n, w, k, stride, y, proj = args
    keep, wp = _w(k)
    got = B.lib().sys_conv1d_strided(x, n, wp if w else None, k, stride, y, proj, None)
    assert got == want, B.status_string(got)


def test_conv1d_strided_has():
    for k in (1, 2, 5, 16, 64):
        assert B.sys_conv1d_strided_has("AUTO", k, 2) and B.sys_conv1d_strided_has("FBS", k, 2)
        for proj in ("SBM", "BFS", "BSM", "FSM", "FFS"):
            assert not B.sys_conv1d_strided_has(proj, k, 2)
            assert B.sys_conv1d_strided_has(proj, k, 1) == B.sys_conv1d_has(proj, k)
        assert not B.sys_conv1d_strided_has("FBS", k, 3) and not B.sys_conv1d_strided_has("FBS", k, 0)
    assert not B.sys_conv1d_strided_has("FBS", 65, 2) and not B.sys_conv1d_strided_has("FBS", 0, 2)


@pytest.mark.parametrize("args,want", [
    ((None, 10, 10, 10, "f", 3, 3, 2, Y, 4, 1), B.SYS_ERR_NULL),
    ((X, 10, 10, 10, "f", 3, 3, 2, None, 4, 0), B.SYS_ERR_NULL),
    ((X, 10, 10, 10, "f", 3, 3, 0, Y, 8, 1), B.SYS_ERR_SIZE),
    ((X, 10, 10, 10, "f", 11, 3, 2, Y, 4, 1), B.SYS_ERR_SIZE),
    ((X, 10, 10, 9, "f", 3, 3, 2, Y, 4, 1), B.SYS_ERR_SIZE),
    ((X, 10, 10, 10, "f", 3, 3, 2, Y, 3, 1), B.SYS_ERR_SIZE),            # 4 outputs per row need y_pitch >= 4
    ((X, 100, 100, 100, "f", 16, 3, 2, Y, 50, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, 100, 100, "f", 3, 3, 3, Y, 50, 1), B.SYS_ERR_UNSUPPORTED),  # only strides 1 and 2 are built
    ((X, 100, 100, 100, "f", 3, 3, 2, Y, 50, B.SYS_PROJ_SBM), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, 100, 100, "f", 3, 3, 2, Y, 50, B.SYS_PROJ_BFS), B.SYS_ERR_UNSUPPORTED),
    ((X + 1, 100, 100, 100, "f", 3, 3, 2, Y, 50, 1), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, 100, 100, "f", 3, 3, 2, X + 4 * 5000, 49, 0), B.SYS_ERR_ALIAS),
    ((X, 100, 100, 100, "f", 3, 3, 1, X + 4 * 5000, 98, 1), B.SYS_ERR_ALIAS),   # stride 1 goes through sys_conv2d
])
def test_conv2d_strided_validation(args, want):
    x, h, w, xp, f, kh, kw, stride, y, yp, proj = args
    keep = np.ones(256, np.float32)
    got = B.lib().sys_conv2d_strided(x, h, w, xp, keep.ctypes.data_as(FP) if f else None, kh, kw, stride, y, yp,
                                     proj, None)
    assert got == want, B.status_string(got)


def test_conv2d_strided_has():
    for kh, kw in [(1, 1), (2, 2), (5, 5), (3, 8), (15, 15)]:
        assert B.sys_conv2d_strided_has("AUTO", kh, kw, 2) and B.sys_conv2d_strided_has("FBS", kh, kw, 2)
        for proj in ("SBM", "BFS", "BSM"):
            assert not B.sys_conv2d_strided_has(proj, kh, kw, 2)
            assert B.sys_conv2d_strided_has(proj, kh, kw, 1) == B.sys_conv2d_has(proj, kh, kw)
        assert not B.sys_conv2d_strided_has("FBS", kh, kw, 3) and not B.sys_conv2d_strided_has("FBS", kh, kw, 0)
    assert not B.sys_conv2d_strided_has("FBS", 16, 3, 2)
