"""GPU parity: libsysconv (through its C ABI) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_common import TOL, dev, err1d, err2d, run1d, run2d
from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import workloads as W

pytestmark = pytest.mark.gpu

PROJ_1D = ["FBS", "SBM", "BFS", "BSM", "FSM", "FFS"]
K_1D = [1, 2, 3, 4, 5, 6, 7, 8, 9, 12, 13, 16, 17, 31, 32, 33, 63, 64]


def _sizes_1d(k):
    # n == k (one output), one more, around a register group, around a wavefront's
    # chunk, several workgroups plus a ragged tail
    per_wave = 4 * 4 * (64 - (k + 2) // 4)
    cand = [k, k + 1, k + 3, 255, 256, 257, per_wave - 1, per_wave + k - 1, per_wave + k, 5 * per_wave + 77, 70001]
    return sorted({n for n in cand if n >= k})


@pytest.mark.parametrize("proj", PROJ_1D)
@pytest.mark.parametrize("k", K_1D)
def test_conv1d_random_all_sizes(proj, k):
    for n in _sizes_1d(k):
        x, w = W.random_case(1000 * k + n, (n,), (k,))
        if not B.sys_conv1d_has(proj, k):
            pytest.skip(f"{proj} is not built for k={k}")
        y = run1d(x, w, proj)
        assert y.shape == (n - k + 1,)
        e = err1d(y, x, w)
        assert e <= TOL, f"{proj} k={k} n={n}: rel err {e}"


@pytest.mark.parametrize("proj", PROJ_1D)
@pytest.mark.parametrize("k", [1, 4, 5, 16, 23, 64])
def test_conv1d_integer_data_is_bit_exact(proj, k):
    # small integers: every partial sum is exact in fp32, so any order gives the oracle's bits
    if not B.sys_conv1d_has(proj, k):
        pytest.skip(f"{proj} is not built for k={k}")
    for n in (k, 1000, 33333):
        x, w = W.integer_case(k * 7 + n, (n,), (k,))
        y = run1d(x, w, proj)
        assert np.array_equal(y.astype(np.float64), oracle.conv1d(x, w)), f"{proj} k={k} n={n}"


@pytest.mark.parametrize("proj", PROJ_1D)
def test_conv1d_delta_filter_copies_input(proj):
    x, _ = W.random_case(5, (40000,), (1,))
    for k, j in [(5, 0), (5, 4), (16, 9), (64, 63)]:
        if not B.sys_conv1d_has(proj, k):
            continue
        w = np.zeros(k, np.float32)
        w[j] = 1.0
        y = run1d(x, w, proj)
        assert np.array_equal(y, x[j:j + len(x) - k + 1])


@pytest.mark.parametrize("proj", PROJ_1D)
def test_conv1d_unaligned_pointers_and_guard_bands(proj):
    # x and y start 1..3 floats into their allocations; everything around y must stay untouched
    k, n = 7, 9001
    if not B.sys_conv1d_has(proj, k):
        pytest.skip(f"{proj} is not built for k={k}")
    x, w = W.random_case(77, (n,), (k,))
    for off in (1, 2, 3):
        xbuf = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
        xbuf[off:off + n] = dev(x)
        ybuf = torch.full((n + 64,), float("nan"), dtype=torch.float32, device="cuda")
        yv = ybuf[32 + off: 32 + off + n - k + 1]
        B.sys_conv1d(xbuf[off:off + n], w, yv, projection=proj)
        torch.cuda.synchronize()
        out = ybuf.cpu().numpy()
        assert np.isnan(out[:32 + off]).all() and np.isnan(out[32 + off + n - k + 1:]).all()
        assert err1d(out[32 + off: 32 + off + n - k + 1], x, w) <= TOL


def test_conv1d_adjacent_buffers_are_accepted():
    n, k = 1000, 5
    buf = torch.zeros(2 * n, dtype=torch.float32, device="cuda")
    x, w = W.random_case(3, (n,), (k,))
    buf[:n] = dev(x)
    B.sys_conv1d(buf[:n], w, buf[n:n + n - k + 1], projection="FBS")
    torch.cuda.synchronize()
    assert err1d(buf[n:n + n - k + 1].cpu().numpy(), x, w) <= TOL
    with pytest.raises(B.SysconvError) as ei:
        B.sys_conv1d(buf[:n], w, buf[n - 1:n - 1 + n - k + 1], projection="FBS")
    assert ei.value.status == B.SYS_ERR_ALIAS


# ------------------------------------------------------------------- 2-D
SHAPES_2D = [(1, 1), (1, 5), (5, 1), (2, 2), (3, 3), (4, 4), (5, 5), (6, 6), (7, 7), (8, 8), (9, 9), (10, 10), (11, 11), (12, 12), (15, 15), (3, 8), (8, 3), (4, 13)]


def _images(kh, kw):
    cols = 4 * (64 - (kw + 2) // 4)          # output columns per strip
    cand = [(kh, kw), (kh + 1, kw + 2), (40, 300), (33 + kh, cols + kw - 1), (70, cols + kw), (129, 2 * cols + 5), (257, 531)]
    return [(h, w) for h, w in cand if h >= kh and w >= kw]


def _projs_2d(kh, kw):
    return [p for p in ("FBS", "BFS", "SBM") if B.sys_conv2d_has(p, kh, kw)]


@pytest.mark.parametrize("kshape", SHAPES_2D)
def test_conv2d_random_all_sizes(kshape):
    kh, kw = kshape
    for proj in _projs_2d(kh, kw):
        for (h, w) in _images(kh, kw):
            x, f = W.random_case(h * 1000 + w + kh, (h, w), (kh, kw), x_range=(0.0, 1.0))
            y = run2d(x, f, proj)
            assert y.shape == (h - kh + 1, w - kw + 1)
            e = err2d(y, x, f)
            assert e <= TOL, f"{proj} {kh}x{kw} image {h}x{w}: rel err {e}"


@pytest.mark.parametrize("k", range(2, 12))
def test_conv2d_single_row_and_single_column_filters(k):
    # 1 x k and k x 1 (the two passes of a separable filter) run kernels of their own: strips of 4 * (64 - halo) columns,
    # rounded down to whole 64-byte pieces for single rows, 16 output rows per workgroup
    for (kh, kw) in [(1, k), (k, 1)]:
        strip = 4 * ((64 - (kw + 2) // 4) & ~3 if kh == 1 else 64)
        for (h, w) in [(kh, kw), (kh + 15, kw + strip - 1), (kh + 16, kw + strip), (kh + 33, kw + 2 * strip + 3), (131, 1031)]:
            x, f = W.random_case(h * 100 + w + k, (h, w), (kh, kw), x_range=(0.0, 1.0))
            for proj in ("FBS", "AUTO"):
                y = run2d(x, f, proj)
                assert y.shape == (h - kh + 1, w - kw + 1)
                e = err2d(y, x, f)
                assert e <= TOL, f"{proj} {kh}x{kw} image {h}x{w}: rel err {e}"
        xi, fi = W.integer_case(k, (70, 600), (kh, kw), x_max=9, w_max=5)
        assert np.array_equal(run2d(xi, fi, "FBS").astype(np.float64), oracle.conv2d(xi, fi)), f"{kh}x{kw}"


@pytest.mark.parametrize("kh", range(2, 12))
def test_conv2d_every_rectangular_filter_with_a_compile_time_kernel(kh):
    # all kh x kw up to 11 x 11 whose smaller side is at most 7 have an FBS kernel sized at compile time (2 output
    # rows per wavefront up to 5 filter rows, 4 from 6 on: workgroups of 8 or 16 output rows); one image with a
    # ragged last tile and strip each
    for kw in range(2, 12 if kh <= 7 else 8):
        cols = 4 * (64 - (kw + 2) // 4)
        for (h, w) in [(kh + 16, kw + cols), (kh + 41, 2 * cols + kw + 2)]:
            x, f = W.random_case(h * 77 + w + 13 * kh + kw, (h, w), (kh, kw), x_range=(-1.0, 1.0))
            y = run2d(x, f, "FBS")
            e = err2d(y, x, f)
            assert e <= TOL, f"FBS {kh}x{kw} image {h}x{w}: rel err {e}"
        xi, fi = W.integer_case(10 * kh + kw, (50, 600), (kh, kw), x_max=9, w_max=5)
        assert np.array_equal(run2d(xi, fi, "FBS").astype(np.float64), oracle.conv2d(xi, fi)), f"{kh}x{kw}"


@pytest.mark.parametrize("kk", [2, 3, 5, 6, 7, 8, 9, 11])
def test_conv2d_tall_images_cover_every_item_height(kk):
    # The strip kernels give a wavefront 2 ... 16 output rows, fewer on images that would not yield 4096
    # items otherwise.  Tall, narrow images (one strip) with 2, 4, 8 and 16 times 4096 rows (+ a ragged
    # rest) make every height run, ring wrap-around and last short item included.
    for mult in (2, 4, 8, 16):
        oh, ow = mult * 4096 + 5, 37
        h, w = oh + kk - 1, ow + kk - 1
        x, f = W.random_case(mult * 100 + kk, (h, w), (kk, kk), x_range=(0.0, 1.0))
        for proj in ("BFS", "SBM"):
            y = run2d(x, f, proj)
            e = err2d(y, x, f)
            assert e <= TOL, f"{proj} {kk}x{kk} image {h}x{w}: rel err {e}"


@pytest.mark.parametrize("kshape", [(2, 2), (3, 3), (5, 5), (11, 11), (4, 6)])
def test_conv2d_integer_data_is_bit_exact(kshape):
    kh, kw = kshape
    for proj in _projs_2d(kh, kw):
        x, f = W.integer_case(kh * 31 + kw, (150, 700), (kh, kw), x_max=9, w_max=5)
        y = run2d(x, f, proj)
        assert np.array_equal(y.astype(np.float64), oracle.conv2d(x, f)), f"{proj} {kh}x{kw}"


def test_conv2d_pitched_views_and_guard_bands():
    # image and result are windows inside larger allocations with odd pitches
    for (kh, kw) in [(3, 3), (5, 5), (6, 2)]:
        for proj in _projs_2d(kh, kw):
            h, w = 61, 523
            x, f = W.random_case(9 + kh, (h, w), (kh, kw), x_range=(0.0, 1.0))
            xbig = torch.zeros((h + 2, w + 13), dtype=torch.float32, device="cuda")
            xbig[1:1 + h, 5:5 + w] = dev(x)
            oh, ow = h - kh + 1, w - kw + 1
            ybig = torch.full((oh + 4, ow + 11), float("nan"), dtype=torch.float32, device="cuda")
            B.sys_conv2d(xbig[1:1 + h, 5:5 + w], f, ybig[2:2 + oh, 3:3 + ow], projection=proj)
            torch.cuda.synchronize()
            out = ybig.cpu().numpy()
            inner = out[2:2 + oh, 3:3 + ow].copy()
            out[2:2 + oh, 3:3 + ow] = np.nan
            assert np.isnan(out).all(), f"{proj} {kh}x{kw} wrote outside its output window"
            assert err2d(inner, x, f) <= TOL, f"{proj} {kh}x{kw}"


def test_conv2d_delta_filter_copies_image():
    x, _ = W.random_case(6, (90, 600), (1, 1), x_range=(0.0, 1.0))
    for (kh, kw, p, q) in [(3, 3, 2, 1), (5, 5, 0, 4), (11, 11, 10, 10), (4, 7, 3, 0)]:
        f = np.zeros((kh, kw), np.float32)
        f[p, q] = 1.0
        for proj in _projs_2d(kh, kw):
            y = run2d(x, f, proj)
            assert np.array_equal(y, x[p:p + 90 - kh + 1, q:q + 600 - kw + 1]), f"{proj} {kh}x{kw}"


def test_auto_projection_runs_everywhere():
    x, w = W.random_case(1, (5000,), (9,))
    assert err1d(run1d(x, w, "AUTO"), x, w) <= TOL
    for kshape in [(4, 4), (5, 5)]:
        img, f = W.random_case(2, (64, 300), kshape)
        assert err2d(run2d(img, f, "AUTO"), img, f) <= TOL


def test_copy_kernel():
    for n in (1, 3, 4096, 4097, 1 << 20):
        a = torch.randn(n, device="cuda")
        b = torch.zeros(n + 2, device="cuda")
        B.sys_copy_f32(a, b[:n])
        torch.cuda.synchronize()
        assert torch.equal(a, b[:n]) and float(b[n:].abs().sum()) == 0.0


def test_alu_yardstick_runs_and_counts_its_multiply_adds():
    out = torch.full((4 * 256 + 8,), float("nan"), dtype=torch.float32, device="cuda")
    n = B.sys_alu_yardstick_f32(out[:4 * 256], 4, 3)
    torch.cuda.synchronize()
    assert n == 4 * 256 * 3 * 256
    res = out.cpu().numpy()
    assert np.isfinite(res[:4 * 256]).all() and np.isnan(res[4 * 256:]).all()
    # every workgroup does the same arithmetic: lane l of each holds the same value
    assert np.array_equal(res[:256], res[256:512]) and np.array_equal(res[:256], res[768:1024])
    with pytest.raises(ValueError):
        B.sys_alu_yardstick_f32(out[:100], 4, 3)


def test_runs_on_a_side_stream():
    s = torch.cuda.Stream()
    x, w = W.random_case(4, (100000,), (16,))
    dx = dev(x)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        y = B.sys_conv1d(dx, w, projection="FBS")           # binding picks up torch's current stream
    s.synchronize()
    assert err1d(y.cpu().numpy(), x, w) <= TOL
