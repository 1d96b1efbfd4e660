"""GPU parity on seeded random shapes: every projection of both convolutions, pitched views, rows long
enough for the banded work order (pitch >= 32 KB), image heights around the item heights."""
import numpy as np
import pytest
import torch

from gpu_common import TOL, dev, err1d, err2d
from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import workloads as W

pytestmark = pytest.mark.gpu


def _conv2d_pitched(x, f, proj, x_pad, y_pad):
    h, w = x.shape
    kh, kw = f.shape
    xb = torch.zeros((h, w + x_pad), dtype=torch.float32, device="cuda")
    xb[:, :w] = dev(x)
    yb = torch.full((h - kh + 1, w - kw + 1 + y_pad), float("nan"), dtype=torch.float32, device="cuda")
    B.sys_conv2d(xb[:, :w], f, yb[:, :w - kw + 1], projection=proj)
    torch.cuda.synchronize()
    out = yb.cpu().numpy()
    assert np.isnan(out[:, w - kw + 1:]).all(), "wrote into the pitch padding"
    return out[:, :w - kw + 1]


@pytest.mark.parametrize("seed", range(40))
def test_conv2d_random_small_shapes(seed):
    rng = np.random.default_rng(7000 + seed)
    kh, kw = (int(rng.integers(1, 16)), int(rng.integers(1, 16))) if seed % 3 == 0 else (int(rng.integers(2, 12)),) * 2
    h = kh + int(rng.integers(0, 300))
    w = kw + int(rng.integers(0, 900))
    x, f = W.random_case(seed, (h, w), (kh, kw), x_range=(0.0, 1.0))
    for proj in ("AUTO", "FBS", "BFS", "SBM"):
        if not B.sys_conv2d_has(proj, kh, kw):
            continue
        y = _conv2d_pitched(x, f, proj, int(rng.integers(0, 9)), int(rng.integers(0, 9)))
        e = err2d(y, x, f)
        assert e <= TOL, f"seed {seed} {proj} {kh}x{kw} image {h}x{w}: rel err {e}"


@pytest.mark.parametrize("seed", range(24))
def test_conv2d_random_long_rows_use_the_banded_order(seed):
    # pitch >= 8192 floats switches the work order to bands of 16 strips; widths chosen so that the strip
    # count is below, equal to and above multiples of 16, heights so that row blocks are ragged
    rng = np.random.default_rng(8000 + seed)
    kk = int(rng.integers(2, 12))
    strips = int(rng.choice([31, 32, 33, 35, 47, 48, 49, 64]))
    ow = strips * 252 - int(rng.integers(0, 252))
    w = max(ow + kk - 1, 8192)
    h = kk + int(rng.integers(0, 70))
    x, f = W.random_case(100 + seed, (h, w), (kk, kk), x_range=(0.0, 1.0))
    for proj in ("FBS", "BFS", "SBM"):
        y = _conv2d_pitched(x, f, proj, int(rng.integers(0, 5)), int(rng.integers(0, 5)))
        e = err2d(y, x, f)
        assert e <= TOL, f"seed {seed} {proj} {kk}x{kk} image {h}x{w}: rel err {e}"


@pytest.mark.parametrize("seed", range(30))
def test_conv1d_random_shapes_all_entry_points(seed):
    rng = np.random.default_rng(9000 + seed)
    k = int(rng.integers(1, 65))
    n = k + int(rng.integers(0, 200000))
    x, w = W.random_case(200 + seed, (n,), (k,))
    dx = dev(x)
    for proj in ("AUTO", "FBS", "SBM", "BFS", "BSM", "FSM", "FFS"):
        y = B.sys_conv1d(dx, w, projection=proj).cpu().numpy()
        e = err1d(y, x, w)
        assert e <= TOL, f"seed {seed} {proj} k={k} n={n}: rel err {e}"
    y2 = B.sys_conv1d_strided(dx, w, 2, projection="FBS").cpu().numpy()
    full = B.sys_conv1d(dx, w, projection="FBS").cpu().numpy()
    import oracle
    ref = oracle.conv1d_strided(x, w, 2, 16)
    scale = oracle.absdot1d_strided(x, w, 2, 16)
    assert oracle.max_rel_err(y2, ref, scale) <= TOL, f"seed {seed} stride 2 k={k} n={n}"
    assert y2.shape == full[::2].shape
    if k <= 16:
        for name in ("FBS", "FSM", "FFS"):
            ys = B.sys_conv1d_stt(dx[:min(n, k + 5000)], w, B.named_design(name)).cpu().numpy()
            assert err1d(ys, x[:min(n, k + 5000)], w) <= TOL, f"seed {seed} generic {name}"
