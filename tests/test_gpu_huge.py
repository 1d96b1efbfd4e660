"""GPU parity at the sizes of the benchmark's paper-shaped grid (671 M outputs per case: inputs and
outputs of 2.7 - 5.4 GB, byte offsets beyond 2^32).  The oracle cannot sweep such a case in seconds, so it
recomputes sampled outputs: whole contiguous pieces (both ends and the places where byte offsets pass 2^31,
2^32 and 2^33) and some twenty thousand single outputs whose input windows are copied to the host, from the
very inputs the kernel read."""
import numpy as np
import pytest
import torch

import oracle
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


def _oracle_on_windows_1d(win, w):
    """One output per gathered window, through the oracle's own routines: the windows laid end to end are a
    signal whose outputs at stride k are exactly the windows' sums."""
    k = len(w)
    flat = np.ascontiguousarray(win, dtype=np.float32).reshape(-1)
    return oracle.conv1d_strided(flat, w, k), oracle.absdot1d_strided(flat, w, k)


def _oracle_on_windows_2d(win, f):
    """The same for kh x kw windows: stacked on top of each other they are an image kw wide whose
    outputs at stride kh (one column) are the windows' sums."""
    kh, kw = f.shape
    img = np.ascontiguousarray(win, dtype=np.float32).reshape(-1, kw)
    if kh == kw:
        return oracle.conv2d_strided(img, f, kh)[:, 0], oracle.absdot2d_strided(img, f, kh)[:, 0]
    raise NotImplementedError


def _check_1d(x, y, w, stride, rng, what):
    k = len(w)
    m = y.shape[0]
    # contiguous pieces: the oracle runs over slices of the device's input
    pieces = [0, m - 4096] + [b // 4 - 2048 for b in (1 << 31, 1 << 32, 1 << 33) if b // 4 + 2048 < m]
    for c0 in pieces:
        c1 = c0 + 4096
        xs = x[stride * c0:stride * (c1 - 1) + k].cpu().numpy()
        ref = oracle.conv1d_strided(xs, w, stride)
        scale = oracle.absdot1d_strided(xs, w, stride)
        err = oracle.max_rel_err(y[c0:c1].cpu().numpy(), ref, scale)
        assert err <= TOL, f"{what}: outputs {c0}..{c1}: rel err {err}"
    # scattered single outputs
    c = torch.from_numpy(_sample_1d(m, rng)).cuda()
    win = x[(stride * c)[:, None] + torch.arange(k, device="cuda")[None, :]].cpu().numpy()
    ref, scale = _oracle_on_windows_1d(win, w)
    got = y[c].cpu().numpy().astype(np.float64)
    bad = np.abs(got - ref) > TOL * scale
    assert not bad.any(), f"{what}: {int(bad.sum())} of {len(bad)} sampled outputs off, first at c={int(c[bad.argmax()])}"


def _check_2d(x, y, f, stride, rng, special_rows, what):
    kk = f.shape[0]
    oh, ow = y.shape
    # contiguous pieces: top-left and bottom-right corners and a band around each special row
    for r0, c0 in [(0, 0), (oh - 24, ow - 300)] + [(r - 12, c) for r in special_rows for c in (0, ow - 300)]:
        r1, c1 = r0 + 24, c0 + 300
        xs = x[stride * r0:stride * (r1 - 1) + kk, stride * c0:stride * (c1 - 1) + kk].cpu().numpy()
        ref = oracle.conv2d_strided(xs, f, stride)
        scale = oracle.absdot2d_strided(xs, f, stride)
        err = oracle.max_rel_err(y[r0:r1, c0:c1].cpu().numpy(), ref, scale)
        assert err <= TOL, f"{what}: rows {r0}..{r1} columns {c0}..{c1}: rel err {err}"
    rows = np.concatenate([np.arange(0, 12), np.arange(oh - 12, oh), rng.integers(0, oh, 3000)]
                          + [np.full(200, r) for r in special_rows])
    cols = np.concatenate([rng.integers(0, ow, len(rows) - 400), np.arange(0, 100), np.arange(ow - 100, ow),
                           rng.integers(0, ow, 200)])
    r = torch.from_numpy(rows).cuda()
    c = torch.from_numpy(cols).cuda()
    ar = torch.arange(kk, device="cuda")
    win = x[(stride * r[:, None, None] + ar[None, :, None]), (stride * c[:, None, None] + ar[None, None, :])]
    ref, scale = _oracle_on_windows_2d(win.cpu().numpy(), f)
    got = y[r, c].cpu().numpy().astype(np.float64)
    bad = np.abs(got - ref) > TOL * scale
    assert not bad.any(), f"{what}: {int(bad.sum())} sampled outputs off, first at {rows[bad.argmax()]},{cols[bad.argmax()]}"


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
    _check_2d(x, y, f, 1, rng, [13107, 13108], f"{proj} {kk}x{kk}")    # row 13107 x 40964 x 4 B crosses 2^31 bytes


@pytest.mark.parametrize("kk", [2, 5])
def test_2d_paper_shape_stride2(kk):
    rng = np.random.default_rng(60 + kk)
    f = rng.uniform(-1, 1, (kk, kk)).astype(np.float32)
    oh, ow = 16384, OUTPUTS // 16384
    x = _uniform((2 * (oh - 1) + kk, 2 * (ow - 1) + kk), 158849)          # 10.7 GB: offsets beyond 2^33 bytes
    y = B.sys_conv2d_strided(x, f, 2, projection="FBS")
    torch.cuda.synchronize()
    assert y.shape == (oh, ow)
    _check_2d(x, y, f, 2, rng, [6553, 13107], f"stride 2 {kk}x{kk}")   # rows around 2^32 and 2^33 bytes of input
    del x, y
    torch.cuda.empty_cache()
