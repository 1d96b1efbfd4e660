"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.
The oracle computes every output (it is threaded), so the comparison is exhaustive."""
import numpy as np
import pytest
import torch

import oracle
from gpu_common import ORACLE_THREADS, TOL, dev, run1d, run2d
from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["conv1d_64k_k5", "conv1d_64m_k16"])
def test_1d_workloads(name):
    wl = W.WORKLOADS[name]
    x, w = W.make(wl)
    ref = oracle.conv1d(x, w, ORACLE_THREADS)
    scale = oracle.absdot1d(x, w, ORACLE_THREADS)
    for proj in ("FBS", "SBM", "BFS", "BSM", "FSM", "FFS"):
        if not B.sys_conv1d_has(proj, len(w)):
            continue
        y = run1d(x, w, proj)
        e = oracle.max_rel_err(y, ref, scale)
        print(f"{name} {proj}: max rel err {e:.3e}", flush=True)
        assert e <= TOL, f"{name} {proj}: {e}"


@pytest.mark.parametrize("name", ["conv2d_1k_3x3", "conv2d_4k_5x5", "conv2d_8k_11x11"])
def test_2d_workloads(name):
    wl = W.WORKLOADS[name]
    x, f = W.make(wl)
    ref = oracle.conv2d(x, f, ORACLE_THREADS)
    scale = oracle.absdot2d(x, f, ORACLE_THREADS)
    for proj in ("FBS", "BFS", "SBM"):
        if not B.sys_conv2d_has(proj, *wl.k_shape):
            continue
        y = run2d(x, f, proj)
        e = oracle.max_rel_err(y, ref, scale)
        print(f"{name} {proj}: max rel err {e:.3e}", flush=True)
        assert e <= TOL, f"{name} {proj}: {e}"


def test_separable_5x5_equals_two_1d_passes_on_the_gpu():
    # 4096 x 4096, f = u v^T: rows with v, then columns with u (via a transpose), all on the
    # GPU path; compared with the direct 2-D GPU result and with the oracle.
    wl = W.WORKLOADS["conv2d_4k_5x5"]
    x, u, v = W.make_separable(wl)
    f = np.outer(u.astype(np.float64), v.astype(np.float64)).astype(np.float32)
    y2 = run2d(x, f, "AUTO")
    dx = dev(x)
    rows = B.sys_conv2d(dx, v[None, :], projection="FBS")                   # 1 x 5 filter
    both = B.sys_conv2d(rows, u[:, None], projection="FBS")                 # 5 x 1 filter
    torch.cuda.synchronize()
    both = both.cpu().numpy()
    scale = oracle.absdot2d(x, np.abs(f), ORACLE_THREADS)
    # f was rounded to fp32 after the outer product (<= 2^-24 relative per tap), and the
    # two-pass route rounds the intermediate image once more: allow 3 ulp-of-scale on top
    assert oracle.max_rel_err(both, y2.astype(np.float64), scale) <= TOL
    ref = oracle.conv2d(x, f, ORACLE_THREADS)
    assert oracle.max_rel_err(y2, ref, scale) <= TOL
