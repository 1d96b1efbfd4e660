"""GPU parity of the stride-2 2-D FBS kernel against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_common import ORACLE_THREADS, TOL, dev
from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import workloads as W

pytestmark = pytest.mark.gpu

KSHAPES = [(1, 1), (1, 2), (2, 1), (2, 2), (3, 3), (4, 4), (5, 5), (6, 6), (7, 7), (8, 8), (9, 9), (11, 11), (15, 15),
           (3, 8), (8, 3), (1, 15), (15, 1), (4, 13)]


def run(x, f, proj="FBS"):
    y = B.sys_conv2d_strided(dev(x), f, 2, projection=proj)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def err(y, x, f):
    ref = oracle.conv2d_strided(x, f, 2, ORACLE_THREADS)
    scale = oracle.absdot2d_strided(x, f, 2, ORACLE_THREADS)
    return oracle.max_rel_err(y, ref, scale)


def _images(kh, kw):
    cols = 4 * (64 - ((kw + 1) // 2 + 2) // 4)           # output columns of a tile
    cand = [(kh, kw), (kh + 1, kw + 1), (kh + 2, kw + 3), (41, 301), (40, 300), (2 * 8 + kh - 2, 2 * cols + kw - 2),
            (2 * 8 + kh - 1, 2 * cols + kw - 1), (2 * 8 + kh, 2 * cols + kw), (2 * 17 + kh, 4 * cols + kw + 7), (259, 1533)]
    return [(h, w) for h, w in cand if h >= kh and w >= kw]


@pytest.mark.parametrize("proj", ["FBS", "AUTO"])
@pytest.mark.parametrize("kshape", KSHAPES)
def test_stride2_2d_random_all_sizes(kshape, proj):
    kh, kw = kshape
    for (h, w) in _images(kh, kw):
        x, f = W.random_case(h * 1000 + w + kh, (h, w), (kh, kw), x_range=(0.0, 1.0))
        y = run(x, f, proj)
        assert y.shape == ((h - kh) // 2 + 1, (w - kw) // 2 + 1)
        e = err(y, x, f)
        assert e <= TOL, f"{kh}x{kw} image {h}x{w}: rel err {e}"


@pytest.mark.parametrize("kshape", [(2, 2), (3, 3), (5, 5), (11, 11), (4, 7)])
def test_stride2_2d_integer_data_is_bit_exact(kshape):
    kh, kw = kshape
    for shape in [(150, 700), (151, 701), (33, 1100)]:
        x, f = W.integer_case(kh * 31 + kw + shape[0], shape, (kh, kw), x_max=9, w_max=5)
        y = run(x, f)
        assert np.array_equal(y.astype(np.float64), oracle.conv2d_strided(x, f, 2)), f"{kh}x{kw} {shape}"


def test_stride2_2d_delta_filter_picks_every_second_pixel():
    x, _ = W.random_case(6, (91, 603), (1, 1), x_range=(0.0, 1.0))
    for (kh, kw, p, q) in [(1, 1, 0, 0), (3, 3, 2, 1), (5, 5, 0, 4), (5, 5, 4, 3), (11, 11, 10, 10), (4, 7, 3, 0), (2, 15, 1, 14)]:
        f = np.zeros((kh, kw), np.float32)
        f[p, q] = 1.0
        y = run(x, f)
        assert np.array_equal(y, x[p:p + 2 * y.shape[0]:2, q:q + 2 * y.shape[1]:2]), (kh, kw, p, q)


def test_stride2_2d_is_every_second_output_of_stride1_on_integer_data():
    x, f = W.integer_case(77, (300, 900), (5, 5), x_max=9, w_max=5)
    y2 = run(x, f)
    y1 = B.sys_conv2d(dev(x), f, projection="FBS").cpu().numpy()
    assert np.array_equal(y2, y1[::2, ::2])


def test_stride1_through_the_strided_entry_is_sys_conv2d():
    x, f = W.random_case(3, (200, 500), (5, 5), x_range=(0.0, 1.0))
    for proj in ("AUTO", "FBS", "SBM", "BFS"):
        a = B.sys_conv2d_strided(dev(x), f, 1, projection=proj).cpu().numpy()
        b = B.sys_conv2d(dev(x), f, projection=proj).cpu().numpy()
        assert np.array_equal(a, b), proj


def test_stride2_2d_pitched_views_and_guard_bands():
    for (kh, kw) in [(3, 3), (5, 5), (6, 2)]:
        h, w = 61, 1047
        x, f = W.random_case(9 + kh, (h, w), (kh, kw), x_range=(0.0, 1.0))
        xbig = torch.zeros((h + 2, w + 13), dtype=torch.float32, device="cuda")
        xbig[1:1 + h, 5:5 + w] = dev(x)
        oh, ow = (h - kh) // 2 + 1, (w - kw) // 2 + 1
        ybig = torch.full((oh + 4, ow + 11), float("nan"), dtype=torch.float32, device="cuda")
        B.sys_conv2d_strided(xbig[1:1 + h, 5:5 + w], f, 2, ybig[2:2 + oh, 3:3 + ow], projection="FBS")
        torch.cuda.synchronize()
        out = ybig.cpu().numpy()
        inner = out[2:2 + oh, 3:3 + ow].copy()
        out[2:2 + oh, 3:3 + ow] = np.nan
        assert np.isnan(out).all(), f"{kh}x{kw} wrote outside its output window"
        assert err(inner, x, f) <= TOL, f"{kh}x{kw}"


@pytest.mark.parametrize("seed", range(16))
def test_stride2_2d_random_shapes(seed):
    rng = np.random.default_rng(12000 + seed)
    kh, kw = int(rng.integers(1, 16)), int(rng.integers(1, 16))
    if seed % 4 == 0:                                          # long rows: the banded work order
        h, w = kh + int(rng.integers(0, 40)), max(8192, kw) + int(rng.integers(0, 3000))
    else:
        h, w = kh + int(rng.integers(0, 300)), kw + int(rng.integers(0, 1500))
    x, f = W.random_case(300 + seed, (h, w), (kh, kw), x_range=(0.0, 1.0))
    e = err(run(x, f), x, f)
    assert e <= TOL, f"seed {seed} {kh}x{kw} image {h}x{w}: rel err {e}"


def test_stride2_2d_unsupported_requests_launch_nothing():
    x = torch.zeros((100, 100), dtype=torch.float32, device="cuda")
    y = torch.full((60, 60), 7.0, dtype=torch.float32, device="cuda")
    f = np.ones((5, 5), np.float32)
    for proj, stride in [("SBM", 2), ("BFS", 2), ("FBS", 3), ("AUTO", 4)]:
        with pytest.raises(B.SysconvError) as e:
            B.sys_conv2d_strided(x, f, stride, y, projection=proj)
        assert e.value.status == B.SYS_ERR_UNSUPPORTED
    with pytest.raises(B.SysconvError) as e:
        B.sys_conv2d_strided(x, f, 0, y, projection="FBS")
    assert e.value.status == B.SYS_ERR_SIZE
    torch.cuda.synchronize()
    assert (y == 7.0).all()
