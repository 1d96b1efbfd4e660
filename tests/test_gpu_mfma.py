"""GPU parity of the matrix-core projection (SYS_PROJ_MFMA) against the CPU oracle.

Same metric and bound as every other projection, max |y - ref| / sum|f||x| <= 1e-5.  The path multiplies
split fp16 operands (hi + lo, three products, fp32 sums), so on top of the usual cases the tests cover what is
specific to it: the admissible input range |x| < 8, taps of any magnitude, the block structure (4 output rows x
64 columns per instruction group, column groups of 256 outputs fed from units of 2 rows x 272 columns, three
column groups per workgroup, a ring of 4 or 8 operand slots, row blocks sized to the number of CUs), and how
non-finite inputs spread.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_common import ORACLE_THREADS, TOL, dev, err2d, run2d
from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import workloads as W

pytestmark = pytest.mark.gpu

# every filter height 1 .. 13 (they select the kernel instance), widths 1 .. 13, square and not
KSHAPES = [(1, 1), (1, 13), (2, 2), (3, 3), (3, 11), (4, 4), (5, 5), (5, 2), (6, 6), (7, 7), (7, 13), (8, 8), (9, 9),
           (9, 4), (10, 10), (11, 11), (11, 5), (12, 12), (13, 13), (13, 1)]


def _images(kh, kw):
    # one output; a ragged corner; below / at / above one 256-column workgroup and one 64-column strip;
    # heights around multiples of 4 (a step), 8 (the shortest row block) and 64 (the tallest)
    cand = [(kh, kw), (kh + 1, kw + 2), (kh + 3, kw + 62), (kh + 4, kw + 63), (kh + 7, kw + 64), (40, 300),
            (kh + 63, kw + 255), (kh + 64, kw + 256), (kh + 70, kw + 321), (135, 531), (300, 1100)]
    return [(h, w) for h, w in cand if h >= kh and w >= kw]


def test_mfma_is_reported_for_filters_up_to_13():
    for kh in range(1, 16):
        for kw in range(1, 16):
            assert B.sys_conv2d_has("MFMA", kh, kw) == (kh <= 13 and kw <= 13)
    assert not B.sys_conv1d_has("MFMA", 5)
    assert B.projection_name(B.SYS_PROJ_MFMA) == "MFMA"


@pytest.mark.parametrize("kshape", KSHAPES)
def test_mfma_random_all_sizes(kshape):
    kh, kw = kshape
    for (h, w) in _images(kh, kw):
        x, f = W.random_case(h * 1000 + w + kh, (h, w), (kh, kw), x_range=(0.0, 1.0))
        y = run2d(x, f, "MFMA")
        assert y.shape == (h - kh + 1, w - kw + 1)
        e = err2d(y, x, f)
        assert e <= TOL, f"MFMA {kh}x{kw} image {h}x{w}: rel err {e}"


@pytest.mark.parametrize("kk", [1, 3, 5, 8, 11, 13])
def test_mfma_tall_images_cover_every_block_height(kk):
    # The launcher cuts a column of the image into one row block per CU (a multiple of 4 rows, at least 8).
    # Tall, narrow images run blocks of 68 .. 516 rows: many turns of the operand ring and of the 16-slot queue,
    # and a last block that is shorter than the others.
    for oh in (2048 * 8 + 5, 2048 * 16 + 3, 2048 * 32 + 1, 2048 * 64 + 7):
        ow = 37
        h, w = oh + kk - 1, ow + kk - 1
        x, f = W.random_case(oh + kk, (h, w), (kk, kk), x_range=(0.0, 1.0))
        y = run2d(x, f, "MFMA")
        e = err2d(y, x, f)
        assert e <= TOL, f"MFMA {kk}x{kk} image {h}x{w}: rel err {e}"


@pytest.mark.parametrize("kshape", [(1, 1), (3, 1), (3, 2), (3, 3), (8, 5), (11, 11), (13, 13)])
def test_mfma_right_edge_of_the_image(kshape):
    # A column group's unit is 272 input columns: 64 + 4 groups of four, fetched 16 bytes per lane; what is left
    # of a row beyond the last whole group of four (1 .. 3 columns) goes 4 bytes per lane, and nothing is loaded
    # beyond the image.  Widths put the image's edge at every position mod 4 in the 256-column main part and in
    # the 16-column halo part of the last group's unit, leave that group 1, 2 or 3 input columns only, and end
    # the last workgroup (three column groups) after one, two and three groups.
    kh, kw = kshape
    h = kh + 21
    for base in (0, 256, 512, 768, 1536):
        for over in (1, 2, 3, 4, 5, 6, 7, 63, 130, 252, 253, 254, 255, 256):
            ow = base + over                                   # the last group holds `over` output columns
            w = ow + kw - 1
            x, f = W.random_case(1000 * ow + kh, (h, w), (kh, kw), x_range=(0.0, 1.0))
            y = run2d(x, f, "MFMA")
            e = err2d(y, x, f)
            assert e <= TOL, f"MFMA {kh}x{kw} image {h}x{w}: rel err {e}"


@pytest.mark.parametrize("kshape", [(2, 2), (5, 5), (11, 11), (4, 6), (13, 13)])
def test_mfma_integer_data_is_bit_exact(kshape):
    # integers below 8 and small integer taps: both are exact in fp16, every product and partial sum is exact
    kh, kw = kshape
    x, f = W.integer_case(kh * 31 + kw, (150, 700), (kh, kw), x_max=7, w_max=5)
    y = run2d(x, f, "MFMA")
    assert np.array_equal(y.astype(np.float64), oracle.conv2d(x, f)), f"MFMA {kh}x{kw}"


def test_mfma_pitched_views_and_guard_bands():
    for (kh, kw) in [(3, 3), (5, 5), (6, 2), (11, 11)]:
        h, w = 61, 523
        x, f = W.random_case(9 + kh, (h, w), (kh, kw), x_range=(0.0, 1.0))
        for xpad, ypad, xoff, yoff in [(13, 11, 5, 3), (1, 2, 0, 1), (3, 1, 2, 0)]:
            # NaN around the image: reading outside it (beyond the pitch padding too) would spoil the result
            xbig = torch.full((h + 2, w + xpad), float("nan"), dtype=torch.float32, device="cuda")
            xbig[1:1 + h, xoff:xoff + w] = dev(x)
            oh, ow = h - kh + 1, w - kw + 1
            ybig = torch.full((oh + 4, ow + ypad), float("nan"), dtype=torch.float32, device="cuda")
            B.sys_conv2d(xbig[1:1 + h, xoff:xoff + w], f, ybig[2:2 + oh, yoff:yoff + ow], projection="MFMA")
            torch.cuda.synchronize()
            out = ybig.cpu().numpy()
            inner = out[2:2 + oh, yoff:yoff + ow].copy()
            out[2:2 + oh, yoff:yoff + ow] = np.nan
            assert np.isnan(out).all(), f"MFMA {kh}x{kw} wrote outside its output window"
            assert err2d(inner, x, f) <= TOL, f"MFMA {kh}x{kw} pads {xpad},{ypad}"


def test_mfma_delta_filter_reproduces_the_image_to_22_bits():
    x, _ = W.random_case(6, (90, 600), (1, 1), x_range=(0.0, 1.0))
    for (kh, kw, p, q) in [(3, 3, 2, 1), (5, 5, 0, 4), (11, 11, 10, 10), (4, 7, 3, 0), (13, 13, 12, 0)]:
        f = np.zeros((kh, kw), np.float32)
        f[p, q] = 1.0
        y = run2d(x, f, "MFMA")
        want = x[p:p + 90 - kh + 1, q:q + 600 - kw + 1].astype(np.float64)
        # hi + lo keeps 22 significant bits of every input; inputs below 2^-27 count as zero
        assert np.all(np.abs(y - want) <= want * 2.0 ** -21 + 2.0 ** -27), f"MFMA {kh}x{kw}"


def test_mfma_input_range_and_tap_magnitudes():
    # inputs anywhere in (-8, 8); taps spread over six decades, and filters that are tiny or huge as a whole
    rng = np.random.default_rng(99)
    x = rng.uniform(-7.99, 7.99, (120, 700)).astype(np.float32)
    for (kh, kw) in [(5, 5), (11, 11)]:
        for lo_e, hi_e in [(-3, 3), (-29, -27), (25, 29), (0, 0)]:
            f = (rng.uniform(-1, 1, (kh, kw)) * 10.0 ** rng.uniform(lo_e, hi_e, (kh, kw))).astype(np.float32)
            y = run2d(x, f, "MFMA")
            e = err2d(y, x, f)
            assert e <= TOL, f"MFMA {kh}x{kw} taps 1e{lo_e}..1e{hi_e}: rel err {e}"
    # all-zero taps: every output is exactly zero
    y = run2d(x, np.zeros((7, 7), np.float32), "MFMA")
    assert not y.any()
    # filters whose largest tap lies outside [1e-30, 1e30] cannot be scaled into fp16's range: a status, no launch
    dx = dev(x)
    out = torch.full((114, 694), 3.0, dtype=torch.float32, device="cuda")
    for amax in (1e-33, 3e33):
        f = np.full((7, 7), amax, np.float32)
        with pytest.raises(B.SysconvError) as ei:
            B.sys_conv2d(dx, f, out, projection="MFMA")
        assert ei.value.status == B.SYS_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert float(out.min()) == 3.0


def test_mfma_inputs_of_8_or_more_show_up_as_non_finite_outputs():
    x, f = W.random_case(5, (60, 400), (5, 5), x_range=(0.0, 1.0))
    f[np.abs(f) < 0.1] = 0.5
    x[30, 200] = 8.0
    y = run2d(x, f, "MFMA")
    assert not np.isfinite(y[26:31, 196:201]).any()        # the outputs whose window holds the value
    assert np.isfinite(y[:8]).all() and np.isfinite(y[40:]).all()


def test_mfma_nonfinite_inputs_stay_within_the_documented_neighbourhood():
    for (kh, kw) in [(3, 3), (5, 5), (11, 11), (4, 6), (1, 9)]:
        h, w_img = 70, 600
        x, f = W.random_case(kh * 17 + kw, (h, w_img), (kh, kw), x_range=(0.0, 1.0))
        f[np.abs(f) < 0.1] = 0.5
        bad = [(0, 0), (33, 255), (34, 256), (h - 1, w_img - 1), (10, 511)]
        for (r, c) in bad:
            x[r, c] = np.inf
        oh, ow = h - kh + 1, w_img - kw + 1
        covered = np.zeros((oh, ow), bool)
        near = np.zeros((oh, ow), bool)
        for (r, c) in bad:
            covered[max(0, r - kh + 1):min(oh, r + 1), max(0, c - kw + 1):min(ow, c + 1)] = True
            # the blocked sums multiply the value by zero taps for outputs up to 18 rows above / 3 below
            # and 15 columns left / 3 right of it
            near[max(0, r - 18):min(oh, r + 4), max(0, c - 15):min(ow, c + 4)] = True
        y = run2d(x, f, "MFMA")
        assert np.isfinite(y[~near]).all(), f"MFMA {kh}x{kw}: non-finite value leaked further than documented"
        assert (~np.isfinite(y[covered])).all(), f"MFMA {kh}x{kw}: non-finite value lost"
        xs = np.where(np.isfinite(x), x, 0).astype(np.float32)
        ref = oracle.conv2d(xs, f)
        scale = oracle.absdot2d(xs, f)
        assert oracle.max_rel_err(y[~near], ref[~near], scale[~near]) <= TOL


@pytest.mark.parametrize("seed", range(24))
def test_mfma_random_shapes_pitches_and_long_rows(seed):
    rng = np.random.default_rng(12000 + seed)
    kh, kw = int(rng.integers(1, 14)), int(rng.integers(1, 14))
    h = kh + int(rng.integers(0, 300))
    w = kw + int(rng.integers(0, 900)) if seed % 4 else max(kw, 8192 + int(rng.integers(0, 700)))
    x, f = W.random_case(seed, (h, w), (kh, kw), x_range=(-1.0, 1.0))
    xp, yp = int(rng.integers(0, 9)), int(rng.integers(0, 9))
    xb = torch.full((h, w + xp), float("nan"), dtype=torch.float32, device="cuda")
    xb[:, :w] = dev(x)
    yb = torch.full((h - kh + 1, w - kw + 1 + yp), float("nan"), dtype=torch.float32, device="cuda")
    B.sys_conv2d(xb[:, :w], f, yb[:, :w - kw + 1], projection="MFMA")
    torch.cuda.synchronize()
    out = yb.cpu().numpy()
    assert np.isnan(out[:, w - kw + 1:]).all(), "wrote into the pitch padding"
    e = err2d(out[:, :w - kw + 1], x, f)
    assert e <= TOL, f"seed {seed} MFMA {kh}x{kw} image {h}x{w}: rel err {e}"


@pytest.mark.parametrize("name", ["conv2d_1k_3x3", "conv2d_4k_5x5", "conv2d_8k_11x11"])
def test_mfma_full_size_workloads(name):
    wl = W.WORKLOADS[name]
    x, f = W.make(wl)
    ref = oracle.conv2d(x, f, ORACLE_THREADS)
    scale = oracle.absdot2d(x, f, ORACLE_THREADS)
    y = run2d(x, f, "MFMA")
    e = oracle.max_rel_err(y, ref, scale)
    print(f"{name} MFMA: max rel err {e:.3e}", flush=True)
    assert e <= TOL, f"{name} MFMA: {e}"


def test_mfma_chains_on_a_stream_and_in_a_graph():
    h, w_img = 300, 1100
    x, f1 = W.random_case(31, (h, w_img), (11, 11), x_range=(0.0, 1.0))
    f1 *= np.float32(1.0 / 64)                               # keep the intermediate image below 8
    _, f2 = W.random_case(32, (h, w_img), (3, 3), x_range=(0.0, 1.0))
    dx = dev(x)
    mid = torch.zeros((h - 10, w_img - 10), dtype=torch.float32, device="cuda")
    out = torch.zeros((h - 12, w_img - 12), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    B.sys_conv2d(dx, f1, mid, projection="MFMA")
    B.sys_conv2d(mid, f2, out, projection="MFMA")
    torch.cuda.synchronize()
    mid_h = mid.cpu().numpy()
    assert err2d(mid_h, x, f1) <= TOL
    assert err2d(out.cpu().numpy(), mid_h, f2) <= TOL
    # the same two calls recorded by stream capture and replayed on changed inputs
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.sys_conv2d(dx, f1, mid, projection="MFMA")
        B.sys_conv2d(mid, f2, out, projection="MFMA")
    for rep in range(3):
        dx.mul_(0.5 + 0.25 * rep)
        mid.fill_(float("nan"))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        xh = dx.cpu().numpy()
        graph.replay()
        torch.cuda.synchronize()
        mid_h = mid.cpu().numpy()
        assert err2d(mid_h, xh, f1) <= TOL, f"replay {rep}"
        assert err2d(out.cpu().numpy(), mid_h, f2) <= TOL, f"replay {rep}"
