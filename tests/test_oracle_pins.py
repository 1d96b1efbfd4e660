"""Pins for the CPU oracle: things the paper and the mathematics fix.

Each test is chosen so that one plausible mistake in the oracle (a flipped
filter, a transposed operand, a dropped tap, a wrong extent, a pitch mix-up,
fp32 instead of fp64 sums) fails it.  Nothing here touches the GPU path.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _parse_rows(txt):
    rows = [[float(v) for v in row.split()] for row in txt.strip().split(";")]
    return np.array(rows, dtype=np.float32)


def _hand_cases():
    cases = []
    with open(os.path.join(GOLDEN, "hand_sums.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split("|")]
            kind, x, w, y = parts[:4]
            stride = int(parts[4]) if len(parts) > 4 else 1
            if kind in ("1d", "abs1d"):
                cases.append((kind, _parse_rows(x)[0], _parse_rows(w)[0], _parse_rows(y)[0].astype(np.float64), stride))
            else:
                cases.append((kind, _parse_rows(x), _parse_rows(w), _parse_rows(y).astype(np.float64), stride))
    return cases


def _hand_eval(kind, x, w, stride, ora=oracle):
    if kind == "1d":
        return ora.conv1d(x, w)
    if kind == "2d":
        return ora.conv2d(x, w)
    if kind == "abs1d":
        return ora.absdot1d(x, w) if stride == 1 else ora.absdot1d_strided(x, w, stride)
    return ora.absdot2d(x, w) if stride == 1 else ora.absdot2d_strided(x, w, stride)


@pytest.mark.parametrize("case", _hand_cases(), ids=lambda c: f"{c[0]}-{c[1].shape}-{c[2].shape}-s{c[4]}")
def test_hand_expanded_sums(case):
    kind, x, w, y, stride = case
    got = _hand_eval(kind, x, w, stride)
    assert got.shape == y.shape
    assert np.array_equal(got, y)


# ---------------------------------------------------------------- delta filters
@pytest.mark.parametrize("k,j", [(1, 0), (5, 0), (5, 3), (5, 4), (16, 7), (64, 63)])
def test_delta_1d_reproduces_shifted_input(k, j):
    rng = np.random.default_rng(7)
    x = rng.uniform(-1, 1, 300).astype(np.float32)
    w = np.zeros(k, np.float32)
    w[j] = 1.0
    y = oracle.conv1d(x, w)
    assert np.array_equal(y, x[j:j + len(x) - k + 1].astype(np.float64))


@pytest.mark.parametrize("kh,kw,p,q", [(3, 3, 0, 0), (3, 3, 2, 1), (5, 5, 1, 4), (11, 11, 10, 0), (2, 7, 1, 6)])
def test_delta_2d_reproduces_shifted_image(kh, kw, p, q):
    rng = np.random.default_rng(8)
    x = rng.uniform(0, 1, (37, 53)).astype(np.float32)
    f = np.zeros((kh, kw), np.float32)
    f[p, q] = 1.0
    y = oracle.conv2d(x, f)
    oh, ow = 37 - kh + 1, 53 - kw + 1
    assert np.array_equal(y, x[p:p + oh, q:q + ow].astype(np.float64))


# ------------------------------------------------------------------- linearity
def test_linearity_in_taps_and_signal_1d():
    rng = np.random.default_rng(9)
    # multiples of 2^-10 in [-1, 1]: sums and power-of-two multiples stay exact in fp32
    grid = lambda n: (rng.integers(-1024, 1025, n) / 1024.0).astype(np.float32)
    x1, x2 = grid(500), grid(500)
    w1, w2 = grid(16), grid(16)
    a, b = 0.5, -4.0
    wc = (a * w1 + b * w2).astype(np.float32)
    assert np.array_equal(wc.astype(np.float64), a * w1.astype(np.float64) + b * w2.astype(np.float64))
    lhs = oracle.conv1d(x1, wc)
    rhs = a * oracle.conv1d(x1, w1) + b * oracle.conv1d(x1, w2)
    assert np.allclose(lhs, rhs, rtol=0, atol=1e-13)
    xs = (x1 + x2).astype(np.float32)
    assert np.array_equal(xs.astype(np.float64), x1.astype(np.float64) + x2.astype(np.float64))
    assert np.allclose(oracle.conv1d(xs, w1), oracle.conv1d(x1, w1) + oracle.conv1d(x2, w1), rtol=0, atol=1e-13)
    assert np.array_equal(oracle.conv1d((2.0 * x1).astype(np.float32), w1), 2.0 * oracle.conv1d(x1, w1))


def test_linearity_2d():
    rng = np.random.default_rng(10)
    x = rng.uniform(0, 1, (40, 41)).astype(np.float32)
    f1 = rng.integers(-4, 5, (5, 5)).astype(np.float32)
    f2 = rng.integers(-4, 5, (5, 5)).astype(np.float32)
    lhs = oracle.conv2d(x, 2 * f1 - 3 * f2)
    rhs = 2 * oracle.conv2d(x, f1) - 3 * oracle.conv2d(x, f2)
    assert np.allclose(lhs, rhs, rtol=0, atol=1e-12)


# ------------------------------------------------------------------ separable
def test_separable_filter_equals_two_1d_passes():
    rng = np.random.default_rng(11)
    # integer-valued data so both routes are exact and can be compared bit for bit
    x = rng.integers(-9, 10, (33, 47)).astype(np.float32)
    u = rng.integers(-3, 4, 5).astype(np.float32)      # down the rows  (index p)
    v = rng.integers(-3, 4, 4).astype(np.float32)      # along a row    (index q)
    f = np.outer(u, v).astype(np.float32)
    y2 = oracle.conv2d(x, f)
    rows = np.stack([oracle.conv1d(x[r], v) for r in range(x.shape[0])])            # (33, 44)
    rows32 = rows.astype(np.float32)
    assert np.array_equal(rows32.astype(np.float64), rows)
    cols = np.stack([oracle.conv1d(rows32[:, c].copy(), u) for c in range(rows.shape[1])], axis=1)
    assert cols.shape == y2.shape == (29, 44)
    assert np.array_equal(cols, y2)


def test_separable_random_floats():
    rng = np.random.default_rng(12)
    x = rng.uniform(0, 1, (30, 31)).astype(np.float32)
    u = rng.uniform(-1, 1, 5).astype(np.float32)
    v = rng.uniform(-1, 1, 5).astype(np.float32)
    f64 = np.outer(u.astype(np.float64), v.astype(np.float64))
    f = f64.astype(np.float32)
    y2 = oracle.conv2d(x, f)
    # two passes in float64 numpy (rows then columns)
    x64 = x.astype(np.float64)
    rows = sum(v[q].astype(np.float64) * x64[:, q:q + 27] for q in range(5))
    both = sum(u[p].astype(np.float64) * rows[p:p + 26, :] for p in range(5))
    # f was rounded to fp32: bound that perturbation by sum|df||x|
    bound = np.abs(f.astype(np.float64) - f64).sum() * 1.0 + 1e-13
    assert np.max(np.abs(y2 - both)) <= bound


# ---------------------------------------------------------------- closed forms
def test_constant_and_ramp_and_box_closed_forms():
    w = np.array([0.5, -1.25, 2.0, 0.75, -3.0], np.float32)
    n = 200
    ones = np.ones(n, np.float32)
    assert np.array_equal(oracle.conv1d(ones, w), np.full(n - 4, float(w.astype(np.float64).sum())))
    ramp = np.arange(n, dtype=np.float32)
    sw = w.astype(np.float64).sum()
    skw = (np.arange(5) * w.astype(np.float64)).sum()
    assert np.array_equal(oracle.conv1d(ramp, w), np.arange(n - 4) * sw + skw)
    # box filter = difference of prefix sums (integer data: exact)
    rng = np.random.default_rng(13)
    x = rng.integers(-100, 101, n).astype(np.float32)
    box = np.ones(16, np.float32)
    pre = np.concatenate([[0.0], np.cumsum(x.astype(np.float64))])
    assert np.array_equal(oracle.conv1d(x, box), pre[16:] - pre[:-16])


def test_2d_constant_ramp_closed_forms():
    f = np.array([[1, -2, 0.5], [0.25, 4, -1]], np.float32)       # 2 x 3
    h, w = 9, 11
    r, c = np.meshgrid(np.arange(h), np.arange(w), indexing="ij")
    x = (10 * r + c).astype(np.float32)                             # x[r][c] = 10 r + c
    y = oracle.conv2d(x, f)
    f64 = f.astype(np.float64)
    p, q = np.meshgrid(np.arange(2), np.arange(3), indexing="ij")
    rr, cc = np.meshgrid(np.arange(h - 1), np.arange(w - 2), indexing="ij")
    want = (10 * rr + cc) * f64.sum() + (f64 * (10 * p + q)).sum()
    assert np.array_equal(y, want)


# ------------------------------------------------- fp64 accumulation really used
def test_sums_are_taken_in_fp64():
    # 2^24 + 1 is not an fp32 number: an fp32 accumulator would lose the "+1".
    x = np.array([16777216.0, 1.0, 1.0], np.float32)
    w = np.array([1.0, 1.0, 1.0], np.float32)
    assert oracle.conv1d(x, w)[0] == 16777218.0
    x2 = np.array([[16777216.0, 1.0], [1.0, 1.0]], np.float32)
    assert oracle.conv2d(x2, np.ones((2, 2), np.float32))[0, 0] == 16777219.0


# -------------------------------------------------- library routines, float64
@pytest.mark.parametrize("n,k", [(16, 16), (17, 16), (1000, 5), (257, 64), (5, 1)])
def test_against_numpy_correlate_float64(n, k):
    rng = np.random.default_rng(100 + n + k)
    x = rng.uniform(-1, 1, n).astype(np.float32)
    w = rng.uniform(-1, 1, k).astype(np.float32)
    want = np.correlate(x.astype(np.float64), w.astype(np.float64), mode="valid")
    got = oracle.conv1d(x, w)
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("shape,kshape", [((20, 33), (3, 3)), ((64, 50), (5, 5)), ((31, 29), (11, 11)), ((12, 40), (1, 7)), ((40, 12), (7, 1))])
def test_against_torch_conv2d_float64(shape, kshape):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(200 + shape[0])
    x = rng.uniform(0, 1, shape).astype(np.float32)
    f = rng.uniform(-1, 1, kshape).astype(np.float32)
    want = torch.nn.functional.conv2d(torch.from_numpy(x).double()[None, None],
                                      torch.from_numpy(f).double()[None, None])[0, 0].numpy()
    got = oracle.conv2d(x, f)
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=0, atol=1e-12)


def test_against_torch_conv1d_float64():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(300)
    x = rng.uniform(-1, 1, 4099).astype(np.float32)
    w = rng.uniform(-1, 1, 16).astype(np.float32)
    want = torch.nn.functional.conv1d(torch.from_numpy(x).double()[None, None],
                                      torch.from_numpy(w).double()[None, None])[0, 0].numpy()
    assert np.allclose(oracle.conv1d(x, w), want, rtol=0, atol=1e-13)


# ----------------------------------------------------------- brute force, tiny
def test_brute_force_python_loops_tiny():
    rng = np.random.default_rng(14)
    x = rng.uniform(-1, 1, (7, 9)).astype(np.float32)
    f = rng.uniform(-1, 1, (3, 4)).astype(np.float32)
    y = oracle.conv2d(x, f)
    for r in range(5):
        for c in range(6):
            terms = [float(x[r + p, c + q]) * float(f[p, q]) for p in range(3) for q in range(4)]
            z = 0.0
            for t in terms:          # same order as the definition: p outer, q inner
                z += t
            assert y[r, c] == z


# ----------------------------------------------------- thread count is harmless
def test_thread_count_does_not_change_the_result():
    rng = np.random.default_rng(15)
    x = rng.uniform(-1, 1, 10007).astype(np.float32)
    w = rng.uniform(-1, 1, 16).astype(np.float32)
    assert np.array_equal(oracle.conv1d(x, w, nthreads=1), oracle.conv1d(x, w, nthreads=4))
    img = rng.uniform(0, 1, (65, 70)).astype(np.float32)
    f = rng.uniform(-1, 1, (5, 5)).astype(np.float32)
    assert np.array_equal(oracle.conv2d(img, f, nthreads=1), oracle.conv2d(img, f, nthreads=3))


# ------------------------------------------------------------- parity metric
def test_absdot_and_metric():
    x = np.array([1, -2, 3, -4], np.float32)
    w = np.array([-1, 2], np.float32)
    assert np.array_equal(oracle.absdot1d(x, w), np.array([5.0, 8.0, 11.0]))
    img = np.array([[1, -2], [-3, 4]], np.float32)
    assert oracle.absdot2d(img, np.array([[-1, 1], [1, -1]], np.float32))[0, 0] == 10.0
    ref = np.array([1.0, 2.0, 0.0])
    scale = np.array([2.0, 4.0, 0.0])
    assert oracle.max_rel_err(ref, ref, scale) == 0.0
    assert oracle.max_rel_err(ref + np.array([0.0, 4e-5, 0.0]), ref, scale) == pytest.approx(1e-5)
    # a non-zero output where every product is zero can never be right
    assert oracle.max_rel_err(ref + np.array([0.0, 0.0, 1e-30]), ref, scale) == float("inf")
    assert oracle.max_rel_err(np.array([np.nan, 2.0, 0.0]), ref, scale) == float("inf")


# ------------------------------------------- the scale of the metric, sum |x||f|
# The scale is the definition applied to the magnitudes: same windows, same order of the fp64 sums.
# So it must equal conv(|x|, |f|) bit for bit -- with conv pinned above, any indexing mistake in the
# scale routines (transposed window, swapped p and q, pitch taken for width, stride on one axis only) shows.
@pytest.mark.parametrize("n,k,stride", [(300, 5, 1), (257, 16, 1), (64, 64, 1), (301, 7, 2), (302, 6, 3)])
def test_absdot1d_is_the_definition_on_magnitudes(n, k, stride):
    rng = np.random.default_rng(500 + n + k)
    x = rng.uniform(-1, 1, n).astype(np.float32)
    w = rng.uniform(-1, 1, k).astype(np.float32)
    if stride == 1:
        assert np.array_equal(oracle.absdot1d(x, w), oracle.conv1d(np.abs(x), np.abs(w)))
    assert np.array_equal(oracle.absdot1d_strided(x, w, stride), oracle.conv1d_strided(np.abs(x), np.abs(w), stride))


@pytest.mark.parametrize("shape,kshape,stride", [((23, 41), (2, 3), 1), ((40, 19), (5, 2), 1), ((31, 37), (11, 11), 1),
                                                  ((17, 50), (1, 7), 1), ((50, 17), (7, 1), 1), ((26, 45), (3, 5), 2),
                                                  ((45, 26), (4, 2), 3)])
def test_absdot2d_is_the_definition_on_magnitudes(shape, kshape, stride):
    rng = np.random.default_rng(600 + shape[0] + kshape[1])
    x = rng.uniform(-1, 1, shape).astype(np.float32)
    f = rng.uniform(-1, 1, kshape).astype(np.float32)
    if stride == 1:
        assert np.array_equal(oracle.absdot2d(x, f), oracle.conv2d(np.abs(x), np.abs(f)))
    assert np.array_equal(oracle.absdot2d_strided(x, f, stride), oracle.conv2d_strided(np.abs(x), np.abs(f), stride))


class _TransposedScale:
    """A planted mistake, kept on the CPU: the 2-D scale with the window read transposed (x[r+q][c+p]),
    the kind of slip the single symmetric 2x2 value could not see."""
    @staticmethod
    def absdot2d(x, f):
        x64, f64 = np.abs(np.asarray(x, np.float64)), np.abs(np.asarray(f, np.float64))
        kh, kw = f64.shape
        m = max(kh, kw)
        oh, ow = x64.shape[0] - kh + 1, x64.shape[1] - kw + 1
        xp = np.pad(x64, ((0, m), (0, m)))
        return np.array([[sum(xp[r + q, c + p] * f64[p, q] for p in range(kh) for q in range(kw))
                          for c in range(ow)] for r in range(oh)])

    @staticmethod
    def absdot2d_strided(x, f, stride):
        return _TransposedScale.absdot2d(x, f)[::stride, ::stride]


def test_scale_pins_catch_a_transposed_window():
    img = np.array([[1, -2], [-3, 4]], np.float32)
    sym = np.array([[-1, 1], [1, -1]], np.float32)
    assert _TransposedScale.absdot2d(img, sym)[0, 0] == 10.0          # the symmetric case cannot tell
    caught = 0
    for kind, x, w, y, stride in _hand_cases():
        if kind == "abs2d":
            caught += not np.array_equal(_hand_eval(kind, x, w, stride, ora=_TransposedScale), y)
    assert caught == 2                                                  # both hand-expanded scale cases can
    rng = np.random.default_rng(77)
    x = rng.uniform(-1, 1, (12, 15)).astype(np.float32)
    f = rng.uniform(-1, 1, (2, 3)).astype(np.float32)
    assert not np.array_equal(_TransposedScale.absdot2d(x, f), oracle.conv2d(np.abs(x), np.abs(f)))


# ------------------------------------------------- rows further apart than wide
@pytest.mark.parametrize("x_pitch,y_pitch", [(None, 40), (53, None), (61, 37), (48, 36)])
def test_pitched_buffers_give_the_compact_result(x_pitch, y_pitch):
    # 29 x 48 image, 3 x 13 filter -> 27 x 36 outputs.  The padding of the input holds NaN and the gaps of the
    # result a sentinel (the wrapper checks they survive), so taking a pitch for a width, or the input pitch for
    # the output pitch, cannot go unnoticed.
    rng = np.random.default_rng(88)
    x = rng.uniform(-1, 1, (29, 48)).astype(np.float32)
    f = rng.uniform(-1, 1, (3, 13)).astype(np.float32)
    for fn in (oracle.conv2d, oracle.absdot2d):
        want = fn(x, f)
        assert np.all(np.isfinite(want))
        assert np.array_equal(fn(x, f, x_pitch=x_pitch, y_pitch=y_pitch), want)
    for fn in (oracle.conv2d_strided, oracle.absdot2d_strided):
        want = fn(x, f, 2)
        yp = None if y_pitch is None else y_pitch - 18
        assert np.array_equal(fn(x, f, 2, x_pitch=x_pitch, y_pitch=yp), want)
    with pytest.raises(ValueError):
        oracle.conv2d(x, f, x_pitch=47)
    with pytest.raises(ValueError):
        oracle.conv2d(x, f, y_pitch=35)


def test_bad_arguments_raise():
    with pytest.raises(ValueError):
        oracle.conv1d(np.ones(3, np.float32), np.ones(4, np.float32))
    with pytest.raises(ValueError):
        oracle.conv2d(np.ones((3, 3), np.float32), np.ones((4, 1), np.float32))


# -------------------------------------------- planted mistakes must be caught
def test_pins_would_catch_a_flipped_or_transposed_filter():
    # sanity of the pins themselves: a flipped / transposed variant of the
    # definition disagrees with the hand-expanded fixtures.
    x = np.array([1, 2, 4, 8, 16], np.float64)
    w = np.array([3, 0, -1], np.float64)
    flipped = np.convolve(x, w, mode="valid")          # true convolution = flipped taps
    assert not np.array_equal(flipped, np.array([-1.0, -2.0, -4.0]))
    img = np.arange(1, 10, dtype=np.float32).reshape(3, 3)
    f = np.array([[1, 2], [3, 4]], np.float32)
    assert not np.array_equal(oracle.conv2d(img, f.T.copy()), np.array([[37.0, 47.0], [67.0, 77.0]]))


# --------------------------------------------------------------- strided 1-D (Table 2, row 3 right)
def test_strided_hand_sums():
    # y[c] = sum_q x[2c+q] w[q], written out by hand for n = 8, k = 3: c = 0, 1, 2 (2*2+2 = 6 < 8; c = 3 needs x[8]).
    x = np.array([1, -2, 3, 5, -7, 11, 13, -17], np.float32)
    w = np.array([2, -1, 4], np.float32)
    want = np.array([1 * 2 + 2 * 1 + 3 * 4, 3 * 2 - 5 * 1 - 7 * 4, -7 * 2 - 11 * 1 + 13 * 4], np.float64)
    assert np.array_equal(oracle.conv1d_strided(x, w, 2), want)
    # stride 3, k = 2: c = 0, 1, 2 (windows start at 0, 3, 6)
    w2 = np.array([3, 5], np.float32)
    want3 = np.array([1 * 3 - 2 * 5, 5 * 3 - 7 * 5, 13 * 3 - 17 * 5], np.float64)
    assert np.array_equal(oracle.conv1d_strided(x, w2, 3), want3)


@pytest.mark.parametrize("n,k,stride", [(41, 5, 2), (40, 5, 2), (64, 2, 2), (65, 16, 2), (33, 1, 2), (50, 7, 3), (9, 9, 2), (10, 9, 2), (11, 9, 2)])
def test_strided_is_every_stride_th_output_and_length(n, k, stride):
    rng = np.random.default_rng(n * 100 + k)
    x = rng.uniform(-1, 1, n).astype(np.float32)
    w = rng.uniform(-1, 1, k).astype(np.float32)
    y = oracle.conv1d_strided(x, w, stride)
    assert y.shape == ((n - k) // stride + 1,)
    assert np.array_equal(y, oracle.conv1d(x, w)[::stride])          # same fp64 sums in the same order
    lib = np.correlate(x.astype(np.float64), w.astype(np.float64), mode="valid")[::stride]
    assert np.allclose(y, lib, rtol=0, atol=1e-13)
    s = oracle.absdot1d_strided(x, w, stride)
    assert np.array_equal(s, oracle.absdot1d(x, w)[::stride])


def test_strided_stride_one_is_eq2_and_delta_picks_x_2c_plus_j():
    rng = np.random.default_rng(3)
    x = rng.uniform(-1, 1, 100).astype(np.float32)
    w = rng.uniform(-1, 1, 6).astype(np.float32)
    assert np.array_equal(oracle.conv1d_strided(x, w, 1), oracle.conv1d(x, w))
    for j in range(6):
        d = np.zeros(6, np.float32)
        d[j] = 1
        got = oracle.conv1d_strided(x, d, 2)
        assert np.array_equal(got, x[j:j + 2 * len(got):2].astype(np.float64))   # a swapped "2c" / "q" would fail here


def test_strided_bad_arguments():
    x = np.zeros(8, np.float32)
    with pytest.raises(ValueError):
        oracle.conv1d_strided(x, np.zeros(3, np.float32), 0)
    with pytest.raises(ValueError):
        oracle.conv1d_strided(x, np.zeros(9, np.float32), 2)


# --------------------------------------------------------------- strided 2-D
def test_strided_2d_hand_sums():
    # 5 x 6 image 1..30 row-major, f = [[1, 2], [3, 4]], stride 2: outputs at (r, c) = (0..1, 0..2)
    x = np.arange(1, 31, dtype=np.float32).reshape(5, 6)
    f = np.array([[1, 2], [3, 4]], np.float32)
    # window at (2r, 2c): x[2r][2c]*1 + x[2r][2c+1]*2 + x[2r+1][2c]*3 + x[2r+1][2c+1]*4
    want = np.array([[1 + 4 + 21 + 32, 3 + 8 + 27 + 40, 5 + 12 + 33 + 48],
                     [13 + 28 + 57 + 80, 15 + 32 + 63 + 88, 17 + 36 + 69 + 96]], np.float64)
    assert np.array_equal(oracle.conv2d_strided(x, f, 2), want)


@pytest.mark.parametrize("shape,kshape,stride", [((9, 11), (2, 2), 2), ((10, 12), (5, 5), 2), ((11, 13), (5, 5), 2),
                                                  ((8, 20), (3, 1), 2), ((7, 21), (1, 4), 2), ((15, 15), (15, 15), 2),
                                                  ((16, 17), (15, 15), 2), ((13, 19), (3, 5), 3)])
def test_strided_2d_is_the_subsampled_stride1_result(shape, kshape, stride):
    rng = np.random.default_rng(shape[0] * 100 + kshape[1])
    x = rng.uniform(0, 1, shape).astype(np.float32)
    f = rng.uniform(-1, 1, kshape).astype(np.float32)
    y = oracle.conv2d_strided(x, f, stride)
    assert y.shape == ((shape[0] - kshape[0]) // stride + 1, (shape[1] - kshape[1]) // stride + 1)
    assert np.array_equal(y, oracle.conv2d(x, f)[::stride, ::stride])        # same fp64 sums in the same order
    assert np.array_equal(oracle.absdot2d_strided(x, f, stride), oracle.absdot2d(x, f)[::stride, ::stride])
    assert np.array_equal(oracle.conv2d_strided(x, f, 1), oracle.conv2d(x, f))


def test_strided_2d_against_torch_float64_and_deltas():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11)
    x = rng.uniform(0, 1, (23, 31)).astype(np.float32)
    f = rng.uniform(-1, 1, (4, 6)).astype(np.float32)
    lib = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64))[None, None],
                                     torch.from_numpy(f.astype(np.float64))[None, None], stride=2)[0, 0].numpy()
    assert np.allclose(oracle.conv2d_strided(x, f, 2), lib, rtol=0, atol=1e-13)
    for p, q in [(0, 0), (3, 0), (0, 5), (2, 3)]:
        d = np.zeros((4, 6), np.float32)
        d[p, q] = 1
        got = oracle.conv2d_strided(x, d, 2)
        assert np.array_equal(got, x[p:p + 2 * got.shape[0]:2, q:q + 2 * got.shape[1]:2].astype(np.float64))
