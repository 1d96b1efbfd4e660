"""The lane programs of the tap-array kernels (BSM, FSM, FFS), modelled on the CPU,
must compute Eq. 2.  Integer data: every order of summation is exact."""
import numpy as np
import pytest

import oracle
from lane_programs import bsm_wave, ffs_wave, fsm_wave


def _ints(seed, n, k):
    rng = np.random.default_rng(seed)
    return rng.integers(-9, 10, n).astype(np.float32), rng.integers(-5, 6, k).astype(np.float32)


@pytest.mark.parametrize("k", [1, 2, 3, 5, 7, 16, 17, 32, 33, 64])
@pytest.mark.parametrize("seg", [4, 12, 40])
def test_bsm_and_fsm_lane_programs(k, seg):
    arrays = 64 // k
    n_out = arrays * seg
    x, w = _ints(k * 100 + seg, n_out + k - 1, k)
    want = oracle.conv1d(x, w)
    assert np.array_equal(bsm_wave(x, w, seg), want)
    assert np.array_equal(fsm_wave(x, w, seg), want)


@pytest.mark.parametrize("k", [1, 2, 5, 16, 31, 64])
@pytest.mark.parametrize("width", [16, 8, 64])
def test_ffs_lane_program(k, width):
    n_out = (64 // width) * width
    x, w = _ints(k * 7 + width, n_out + k - 1, k)
    assert np.array_equal(ffs_wave(x, w, width), oracle.conv1d(x, w))


# ------------------------------------------------------------------ generic space-time transform
from lane_programs import stt_plan, stt_wave  # noqa: E402
from paper_2010_15884_amd import schedule_model as sm  # noqa: E402

from stt_designs import NOVEL, named as _named  # noqa: E402


@pytest.mark.parametrize("k", [1, 2, 5, 16])
@pytest.mark.parametrize("name", list(sm.TRANSFORMS) + list(NOVEL))
def test_generic_lane_program(name, k):
    alloc, sched, dx, dw, dz = _named(name) if name in sm.TRANSFORMS else NOVEL[name]
    pl = stt_plan(alloc, sched, dx, dw, dz, k)
    for dist in pl["dist"].values():
        assert dist is None or (abs(dist[0]) <= 1 and 1 <= dist[1] <= 3)
    for n_out in (pl["C"], max(1, pl["C"] - 3), 1):               # a full chunk, a ragged one, one output
        x, w = _ints(k * 31 + n_out, n_out + k - 1, k)
        got = stt_wave(alloc, sched, dx, dw, dz, x, w)
        assert np.array_equal(got, oracle.conv1d(x, w)), (name, k, n_out)
