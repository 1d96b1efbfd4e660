"""Host-side checks of the generic space-time-transform entry points (no GPU needed)."""
import ctypes

import numpy as np
import pytest

from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import schedule_model as sm
from stt_designs import INVALID, NOVEL, PAPER, TOO_LARGE

FP = ctypes.POINTER(ctypes.c_float)
X, Y = 0x10000000, 0x40000000          # fake, aligned, non-overlapping device addresses: validation never dereferences them


@pytest.mark.parametrize("k", [1, 2, 5, 16])
def test_the_papers_six_designs_and_the_novel_ones_pass(k):
    for name, d in {**PAPER, **NOVEL}.items():
        assert B.sys_stt_check(B.stt_design(*d), k) == B.SYS_OK, name
    for name in PAPER:
        assert sm.is_valid(name)                                   # the Python model agrees on the paper's six


@pytest.mark.parametrize("name", list(INVALID))
def test_invalid_designs_are_rejected_as_designs(name):
    assert B.sys_stt_check(B.stt_design(*INVALID[name]), 5) == B.SYS_ERR_DESIGN


@pytest.mark.parametrize("name", list(TOO_LARGE))
def test_valid_but_unbuilt_designs_are_unsupported(name):
    assert B.sys_stt_check(B.stt_design(*TOO_LARGE[name]), 5) == B.SYS_ERR_UNSUPPORTED


def test_pe_vector_must_fit_a_wavefront():
    sbm = B.named_design("SBM")                                    # PE = c + q: needs C + k - 1 <= 64 lanes
    assert B.sys_stt_check(sbm, 64) == B.SYS_OK                    # one output per wavefront still fits
    wide = B.stt_design((1, 2), (0, 1), (-1, 1), None, (0, 1))     # PE = c + 2q: P.ex = 1, P.ez = 2 -> far
    assert B.sys_stt_check(wide, 5) == B.SYS_ERR_UNSUPPORTED
    bsm = B.named_design("BSM")                                    # PE = q: k lanes
    assert B.sys_stt_check(bsm, 64) == B.SYS_OK
    assert B.sys_stt_check(bsm, 65) == B.SYS_ERR_SIZE and B.sys_stt_check(bsm, 0) == B.SYS_ERR_SIZE
    assert B.lib().sys_stt_check(None, 5) == B.SYS_ERR_NULL


def test_named_design_matches_the_tables():
    d = B.named_design("FFS")
    assert (list(d.alloc), list(d.sched)) == ([1, 0], [2, 1])
    assert (d.x_passed, list(d.dep_x), d.w_passed, list(d.dep_w), list(d.dep_z)) == (1, [1, -1], 1, [1, 0], [0, 1])
    d = B.named_design("SBM")
    assert (list(d.alloc), list(d.sched), d.x_passed, list(d.dep_x), d.w_passed) == ([1, 1], [0, 1], 1, [-1, 1], 0)


@pytest.mark.parametrize("args,want", [
    ((None, 100, "w", 5, Y, "FBS"), B.SYS_ERR_NULL),
    ((X, 100, None, 5, Y, "FBS"), B.SYS_ERR_NULL),
    ((X, 100, "w", 5, None, "FBS"), B.SYS_ERR_NULL),
    ((X, 100, "w", 5, Y, None), B.SYS_ERR_NULL),
    ((X, 100, "w", 0, Y, "FBS"), B.SYS_ERR_SIZE),
    ((X, 4, "w", 5, Y, "FBS"), B.SYS_ERR_SIZE),
    ((X, 100, "w", 65, Y, "FBS"), B.SYS_ERR_UNSUPPORTED),
    ((X + 2, 100, "w", 5, Y, "FBS"), B.SYS_ERR_UNSUPPORTED),
    ((X, 100, "w", 5, X + 4 * 99, "FBS"), B.SYS_ERR_ALIAS),
    ((X, 100, "w", 5, Y, "singular"), B.SYS_ERR_DESIGN),
    ((X, 100, "w", 5, Y, "det_2"), B.SYS_ERR_UNSUPPORTED),
])
def test_conv1d_stt_validation(args, want):
    x, n, w, k, y, dname = args
    keep = np.ones(max(k, 1), np.float32)
    d = None if dname is None else B.stt_design(*{**PAPER, **INVALID, **TOO_LARGE}[dname])
    got = B.lib().sys_conv1d_stt(x, n, keep.ctypes.data_as(FP) if w else None, k, y,
                                 ctypes.byref(d) if d is not None else None, None)
    assert got == want, B.status_string(got)


def test_extreme_coefficients_are_refused_without_overflow():
    # INT_MIN has no negative and INT_MAX + INT_MAX no sum: the planner must refuse such designs by comparison, not
    # by arithmetic on them (the sanitized build in tests/test_sanitizers.py shows there is no overflow on the way)
    lo, hi = -2 ** 31, 2 ** 31 - 1
    for design in [((hi, 1), (lo, 1), None, None, (0, 1)), ((lo, lo), (hi, hi), (hi, lo), (lo, 0), (0, 1)),
                   ((1, 0), (0, 1), (hi, hi), None, (0, 1)), ((1, 0), (0, 1), (lo, lo), None, (0, 1)),
                   ((1, 0), (1, 1), None, (lo, 0), (0, 1)), ((1, 0), (1, 1), None, None, (0, lo))]:
        got = B.sys_stt_check(B.stt_design(*design), 5)
        assert got in (B.SYS_ERR_UNSUPPORTED, B.SYS_ERR_DESIGN), B.status_string(got)
