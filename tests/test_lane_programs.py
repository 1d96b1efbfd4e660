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
