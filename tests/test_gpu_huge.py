"""GPU parity at the sizes of the benchmark's paper-shaped grid (671 M outputs per case: inputs and
outputs of 2.7 - 5.4 GB, byte offsets beyond 2^32), on sampled outputs that are recomputed one by one
in fp64 on the host from the very inputs the kernel read."""
import numpy as np
import pytest
import torch

from gpu_common import TOL
from paper_2010_15884_amd import binding as B

pytestmark = pytest.mark.gpu

OUTPUTS = 10 * (1 << 20) * 64                     # 10 Mi "threads" x 16*4 outputs (paper Section 6)


def _uniform(shape, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    t = torch.empty(shape, dtype=torch.float32, device="cuda")
    t.uniform_(-1.0, 1.0, generator=g)
    return t


@pytest.fixture(scope="module")
def signal():
    x = _uniform((2 * OUTPUTS + 16,), 158847)
    yield x
    del x
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def image():
    x = _uniform((16384 + 4, OUTPUTS // 16384 + 4), 158848)
    yield x
    del x
    torch.cuda.empty_cache()


def _sample_1d(m, rng):
    special = [0, 1, 255, 256, 1007, 1008, 1 << 29, (1 << 29) + 1, (1 << 30) // 2 - 1, m - 2, m - 1]
    idx = np.concatenate([np.arange(0, 300), np.arange(m - 300, m), np.array([s for s in special if 0 <= s < m]),
                          (1 << 29) + np.arange(-40, 40), rng.integers(0, m, 20000)])
    return np.unique(idx[(idx >= 0) & (idx < m)])


def _check_1d(x, y, w, stride, rng, what):
    k = len(w)
    m = y.shape[0]
    c = torch.from_numpy(_sample_1d(m, rng)).cuda()
    win = x[(stride * c)[:, None] + torch.arange(k, device="cuda")[None, :]].cpu().numpy().astype(np.float64)
    got = y[c].cpu().numpy().astype(np.float64)
    w64 = w.astype(np.float64)
    ref = win @ w64
    scale = np.abs(win) @ np.abs(w64)
    bad = np.abs(got - ref) > TOL * scale
    assert not bad.any(), f"{what}: {int(bad.sum())} of {len(bad)} sampled outputs off, first at c={int(c[bad.argmax()])}"


@pytest.mark.parametrize("k", [2, 5])
@pytest.mark.parametrize("proj", ["AUTO", "FBS", "SBM", "BFS", "BSM", "FSM", "FFS"])
def test_1d_paper_shape_stride1(signal, proj, k):
    rng = np.random.default_rng(k)
    w = rng.uniform(-1, 1, k).astype(np.float32)
    n = OUTPUTS + k - 1
    y = B.sys_conv1d(signal[:n], w, projection=proj)
    torch.cuda.synchronize()
    assert y.shape == (OUTPUTS,)
    _check_1d(signal, y, w, 1, rng, f"{proj} k={k}")


@pytest.mark.parametrize("k", [2, 5, 16])
def test_1d_paper_shape_stride2(signal, k):
    rng = np.random.default_rng(20 + k)
    w = rng.uniform(-1, 1, k).astype(np.float32)
    n = 2 * (OUTPUTS - 1) + k                      # input bytes beyond 2^32
    y = B.sys_conv1d_strided(signal[:n], w, 2, projection="FBS")
    torch.cuda.synchronize()
    assert y.shape == (OUTPUTS,)
    _check_1d(signal, y, w, 2, rng, f"stride 2 k={k}")


@pytest.mark.parametrize("kk", [2, 5])
@pytest.mark.parametrize("proj", ["FBS", "SBM", "BFS"])
def test_2d_paper_shape(image, proj, kk):
    rng = np.random.default_rng(40 + kk)
    f = rng.uniform(-1, 1, (kk, kk)).astype(np.float32)
    oh, ow = 16384, OUTPUTS // 16384
    x = image[:oh + kk - 1, :ow + kk - 1]          # a view: the pitch stays that of the full allocation
    y = B.sys_conv2d(x, f, projection=proj)
    torch.cuda.synchronize()
    assert y.shape == (oh, ow)
    rows = np.concatenate([np.arange(0, 12), np.arange(oh - 12, oh), rng.integers(0, oh, 3000),
                           np.full(200, 13107), np.full(200, 13108)])      # row 13107 x 40964 x 4 B crosses 2^31 bytes
    cols = np.concatenate([rng.integers(0, ow, len(rows) - 400), np.arange(0, 100), np.arange(ow - 100, ow),
                           rng.integers(0, ow, 200)])
    r = torch.from_numpy(rows).cuda()
    c = torch.from_numpy(cols).cuda()
    ar = torch.arange(kk, device="cuda")
    win = x[(r[:, None, None] + ar[None, :, None]), (c[:, None, None] + ar[None, None, :])]
    win = win.cpu().numpy().astype(np.float64).reshape(len(rows), kk * kk)
    got = y[r, c].cpu().numpy().astype(np.float64)
    f64 = f.astype(np.float64).reshape(-1)
    ref = win @ f64
    scale = np.abs(win) @ np.abs(f64)
    bad = np.abs(got - ref) > TOL * scale
    assert not bad.any(), f"{proj} {kk}x{kk}: {int(bad.sum())} sampled outputs off, first at {rows[bad.argmax()]},{cols[bad.argmax()]}"


@pytest.mark.parametrize("kk", [2, 5])
def test_2d_paper_shape_stride2(kk):
    rng = np.random.default_rng(60 + kk)
    f = rng.uniform(-1, 1, (kk, kk)).astype(np.float32)
    oh, ow = 16384, OUTPUTS // 16384
    x = _uniform((2 * (oh - 1) + kk, 2 * (ow - 1) + kk), 158849)          # 10.7 GB: offsets beyond 2^33 bytes
    y = B.sys_conv2d_strided(x, f, 2, projection="FBS")
    torch.cuda.synchronize()
    assert y.shape == (oh, ow)
    rows = np.concatenate([np.arange(0, 12), np.arange(oh - 12, oh), rng.integers(0, oh, 3000),
                           np.full(200, 6553), np.full(200, 13107)])       # rows around 2^32 and 2^33 bytes of input
    cols = np.concatenate([rng.integers(0, ow, len(rows) - 400), np.arange(0, 100), np.arange(ow - 100, ow),
                           rng.integers(0, ow, 200)])
    r = torch.from_numpy(rows).cuda()
    c = torch.from_numpy(cols).cuda()
    ar = torch.arange(kk, device="cuda")
    win = x[(2 * r[:, None, None] + ar[None, :, None]), (2 * c[:, None, None] + ar[None, None, :])]
    win = win.cpu().numpy().astype(np.float64).reshape(len(rows), kk * kk)
    got = y[r, c].cpu().numpy().astype(np.float64)
    f64 = f.astype(np.float64).reshape(-1)
    ref = win @ f64
    scale = np.abs(win) @ np.abs(f64)
    bad = np.abs(got - ref) > TOL * scale
    assert not bad.any(), f"{kk}x{kk}: {int(bad.sum())} sampled outputs off, first at {rows[bad.argmax()]},{cols[bad.argmax()]}"
    del x, y
    torch.cuda.empty_cache()
