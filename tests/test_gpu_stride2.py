"""GPU parity of the stride-2 FBS design (Table 2, row 3 right) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_common import ORACLE_THREADS, TOL, dev
from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import workloads as W

pytestmark = pytest.mark.gpu

K_S2 = [1, 2, 3, 4, 5, 6, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64]


def run_s2(x, w, proj="FBS", stride=2):
    y = B.sys_conv1d_strided(dev(x), w, stride, projection=proj)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def err_s2(y, x, w, stride=2):
    ref = oracle.conv1d_strided(x, w, stride, ORACLE_THREADS)
    scale = oracle.absdot1d_strided(x, w, stride, ORACLE_THREADS)
    return oracle.max_rel_err(y, ref, scale)


def _sizes(k):
    # one output, odd and even n - k, around a register group (256 outputs = 512 inputs), around a
    # wavefront's chunk, several workgroups plus a ragged tail
    per_wave = 4 * 4 * (64 - ((k + 1) // 2 + 2) // 4)
    cand = [k, k + 1, k + 2, k + 3, 511, 512, 513, 2 * per_wave + k - 2, 2 * per_wave + k - 1, 2 * per_wave + k,
            2 * per_wave + k + 1, 10 * per_wave + 155, 140001, 140002]
    return sorted({n for n in cand if n >= k})


@pytest.mark.parametrize("proj", ["FBS", "AUTO"])
@pytest.mark.parametrize("k", K_S2)
def test_stride2_random_all_sizes(proj, k):
    for n in _sizes(k):
        x, w = W.random_case(2000 * k + n, (n,), (k,))
        y = run_s2(x, w, proj)
        assert y.shape == ((n - k) // 2 + 1,)
        e = err_s2(y, x, w)
        assert e <= TOL, f"k={k} n={n}: rel err {e}"


@pytest.mark.parametrize("k", [1, 2, 5, 16, 23, 64])
def test_stride2_integer_data_is_bit_exact(k):
    for n in (k, k + 1, 1000, 33333):
        x, w = W.integer_case(k * 11 + n, (n,), (k,))
        y = run_s2(x, w)
        assert np.array_equal(y.astype(np.float64), oracle.conv1d_strided(x, w, 2)), f"k={k} n={n}"


def test_stride2_delta_filter_picks_every_second_input():
    x, _ = W.random_case(6, (50001,), (1,))
    for k, j in [(1, 0), (2, 1), (5, 0), (5, 3), (5, 4), (16, 9), (64, 63), (64, 62)]:
        w = np.zeros(k, np.float32)
        w[j] = 1.0
        y = run_s2(x, w)
        assert np.array_equal(y, x[j:j + 2 * len(y):2]), (k, j)


def test_stride2_equals_every_second_output_of_stride1_bits():
    # same kernel family, different chains: to rounding only -- but against the oracle both hold, and with
    # integer data the two must agree exactly
    x, w = W.integer_case(99, (70001,), (7,))
    y2 = run_s2(x, w)
    y1 = B.sys_conv1d(dev(x), w, projection="FBS").cpu().numpy()
    assert np.array_equal(y2, y1[::2])


def test_stride1_through_the_strided_entry_is_sys_conv1d():
    x, w = W.random_case(3, (30000,), (9,))
    for proj in ("AUTO", "FBS", "SBM", "BFS", "BSM", "FSM", "FFS"):
        a = B.sys_conv1d_strided(dev(x), w, 1, projection=proj).cpu().numpy()
        b = B.sys_conv1d(dev(x), w, projection=proj).cpu().numpy()
        assert np.array_equal(a, b), proj


def test_stride2_unaligned_pointers_and_guard_bands():
    k, n = 7, 18001
    x, w = W.random_case(78, (n,), (k,))
    m = (n - k) // 2 + 1
    for off in (1, 2, 3):
        xbuf = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
        xbuf[off:off + n] = dev(x)
        ybuf = torch.full((m + 64,), float("nan"), dtype=torch.float32, device="cuda")
        yv = ybuf[32 + off: 32 + off + m]
        B.sys_conv1d_strided(xbuf[off:off + n], w, 2, yv, projection="FBS")
        torch.cuda.synchronize()
        out = ybuf.cpu().numpy()
        assert np.isnan(out[:32 + off]).all() and np.isnan(out[32 + off + m:]).all()
        assert err_s2(out[32 + off: 32 + off + m], x, w) <= TOL


def test_stride2_nonfinite_inputs_stay_local():
    # an Inf or NaN may only reach the outputs whose window covers it (no zero-weight padding may touch it)
    for k in (1, 2, 3, 4, 5, 8, 9, 16, 17, 33, 64):
        n = 6001
        x, w = W.random_case(k + 500, (n,), (k,))
        w[np.abs(w) < 0.1] = 0.5
        bad = {1400: np.inf, 3001: np.nan, n - 1: -np.inf, 0: np.inf}
        for i, v in bad.items():
            x[i] = v
        y = run_s2(x, w)
        m = (n - k) // 2 + 1
        touched = np.zeros(m, bool)
        for i in bad:
            for c in range(max(0, (i - k + 1 + 1) // 2), min(m, i // 2 + 1)):
                if 0 <= i - 2 * c < k:
                    touched[c] = True
        assert np.isfinite(y[~touched]).all(), f"k={k}: non-finite value leaked"
        assert (~np.isfinite(y[touched])).all(), f"k={k}: non-finite value lost"
        xs = np.where(np.isfinite(x), x, 0).astype(np.float32)
        ref = oracle.conv1d_strided(xs, w, 2)
        scale = oracle.absdot1d_strided(xs, w, 2)
        assert oracle.max_rel_err(y[~touched], ref[~touched], scale[~touched]) <= TOL


def test_stride2_large_signal_sampled_against_single_outputs():
    # the size the benchmark's paper-shaped table times; checked on sampled outputs computed one by one
    n, k = (1 << 26) + 5, 5
    x, w = W.random_case(15884, (n,), (k,))
    y = run_s2(x, w)
    m = (n - k) // 2 + 1
    assert y.shape == (m,)
    rng = np.random.default_rng(1)
    idx = np.concatenate([np.arange(0, 64), np.arange(m - 64, m), rng.integers(0, m, 4000)])
    x64, w64 = x.astype(np.float64), w.astype(np.float64)
    for c in idx:
        ref = float(np.dot(x64[2 * c:2 * c + k], w64))
        scale = float(np.dot(np.abs(x64[2 * c:2 * c + k]), np.abs(w64)))
        assert abs(float(y[c]) - ref) <= TOL * scale, c


def test_stride2_unsupported_requests_launch_nothing():
    x = torch.zeros(1000, dtype=torch.float32, device="cuda")
    y = torch.full((600,), 7.0, dtype=torch.float32, device="cuda")
    w = np.ones(5, np.float32)
    for proj, stride in [("SBM", 2), ("BFS", 2), ("FFS", 2), ("FBS", 3), ("AUTO", 4)]:
        with pytest.raises(B.SysconvError) as e:
            B.sys_conv1d_strided(x, w, stride, y, projection=proj)
        assert e.value.status == B.SYS_ERR_UNSUPPORTED
    with pytest.raises(B.SysconvError) as e:
        B.sys_conv1d_strided(x, w, 0, y, projection="FBS")
    assert e.value.status == B.SYS_ERR_SIZE
    torch.cuda.synchronize()
    assert (y == 7.0).all()
