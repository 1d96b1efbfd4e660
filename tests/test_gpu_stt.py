"""GPU parity of the generic space-time-transform kernel against the CPU oracle: the paper's six designs
and designs the paper does not list, all through one kernel."""
import numpy as np
import pytest
import torch

import oracle
from gpu_common import TOL, dev, err1d
from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import workloads as W
from stt_designs import INVALID, NOVEL, PAPER

pytestmark = pytest.mark.gpu

ALL = {**PAPER, **NOVEL}


def run(x, w, name):
    y = B.sys_conv1d_stt(dev(x), w, B.stt_design(*ALL[name]))
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8, 16, 17, 33, 64])
@pytest.mark.parametrize("name", list(ALL))
def test_stt_random_sizes(name, k):
    # one output, a ragged chunk, exactly one and several chunks of every possible chunk length, a long ragged signal
    for n in sorted({k, k + 1, k + 6, 63 + k, 64 + k - 1, 64 + k, 4 * 64 + k - 1, 1000 + k, 30011}):
        x, w = W.random_case(3000 * k + n, (n,), (k,))
        y = run(x, w, name)
        assert y.shape == (n - k + 1,)
        e = err1d(y, x, w)
        assert e <= TOL, f"{name} k={k} n={n}: rel err {e}"


@pytest.mark.parametrize("name", list(ALL))
def test_stt_integer_data_is_bit_exact(name):
    for k in (1, 5, 16):
        for n in (k, 777, 20000):
            x, w = W.integer_case(k * 13 + n, (n,), (k,))
            y = run(x, w, name)
            assert np.array_equal(y.astype(np.float64), oracle.conv1d(x, w)), f"{name} k={k} n={n}"


@pytest.mark.parametrize("name", list(PAPER))
def test_stt_agrees_with_the_hand_laid_projection_on_integer_data(name):
    x, w = W.integer_case(5, (50000,), (5,))
    a = run(x, w, name)
    b = B.sys_conv1d(dev(x), w, projection=name).cpu().numpy()
    assert np.array_equal(a, b)


def test_stt_guard_bands_and_invalid_designs_launch_nothing():
    k, n = 5, 9001
    x, w = W.random_case(79, (n,), (k,))
    ybuf = torch.full((n + 64,), float("nan"), dtype=torch.float32, device="cuda")
    yv = ybuf[32: 32 + n - k + 1]
    B.sys_conv1d_stt(dev(x), w, B.named_design("FSM"), yv)
    torch.cuda.synchronize()
    out = ybuf.cpu().numpy()
    assert np.isnan(out[:32]).all() and np.isnan(out[32 + n - k + 1:]).all()
    assert err1d(out[32: 32 + n - k + 1], x, w) <= TOL
    keep = torch.full((n - k + 1,), 5.0, dtype=torch.float32, device="cuda")
    for name, d in INVALID.items():
        with pytest.raises(B.SysconvError) as e:
            B.sys_conv1d_stt(dev(x), w, B.stt_design(*d), keep)
        assert e.value.status == B.SYS_ERR_DESIGN, name
    torch.cuda.synchronize()
    assert (keep == 5.0).all()
