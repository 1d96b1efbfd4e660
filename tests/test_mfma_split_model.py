"""CPU model of the arithmetic of the matrix-core projection (SYS_PROJ_MFMA), checked against the oracle.

The projection multiplies fp16 numbers and accumulates in fp32.  This file restates that arithmetic in numpy --
scaling by powers of two, the split of every input and tap into hi + lo * 2^-11 (both fp16, rounded to nearest),
the three products hi*hi, lo*hi, hi*lo, one fp32 rounding per instruction (an instruction sums two filter rows),
the cross terms in an accumulator of their own, the final fp32 combination -- and measures what it leaves against
the fp64 definition in the parity metric  max |y - ref| / sum |f||x|.  It is the error study behind the projection's
tolerance: the bound 1e-5 must hold with a margin of three, the cross terms must be needed (hi*hi alone fails), and
without keeping lo 2^11 times larger the fp16 subnormal range (which the matrix cores read as zero) would show.

Nothing here runs on a GPU and nothing is shared with the HIP sources; the model follows the description in
include/sysconv.h (Section 6.2 / Table 5 of the paper motivate the large-filter path).
"""
import numpy as np
import pytest

import oracle
from paper_2010_15884_amd import workloads as W

X_SCALE = 2.0 ** 13
LO_SCALE = 2.0 ** 11
FP16_MIN_NORMAL = 2.0 ** -14


def _tap_scale(f):
    amax = float(np.max(np.abs(f)))
    _, e = np.frexp(amax)                                     # amax = m * 2^e, 0.5 <= m < 1
    return 2.0 ** (14 - int(e))


def _split(v, scale, lo_scale, flush):
    s = v.astype(np.float64) * scale                          # exact: a power of two
    hi = s.astype(np.float16)
    lo = ((s - hi.astype(np.float64)) * lo_scale).astype(np.float16)
    hi, lo = hi.astype(np.float64), lo.astype(np.float64)
    if flush:                                                 # the matrix cores read fp16 subnormals as zero
        hi = np.where(np.abs(hi) < FP16_MIN_NORMAL, 0.0, hi)
        lo = np.where(np.abs(lo) < FP16_MIN_NORMAL, 0.0, lo)
    return hi, lo


def _model(x, f, products=("hh", "lh", "hl"), lo_scale=LO_SCALE, phase=0):
    """The projection's result for image x and filter f.  `phase`: which filter rows share an instruction (the row
    of the output inside its block of four decides it)."""
    kh, kw = f.shape
    oh, ow = x.shape[0] - kh + 1, x.shape[1] - kw + 1
    ts = _tap_scale(f)
    xh, xl = _split(x, X_SCALE, lo_scale, True)
    fh, fl = _split(f, ts, lo_scale, True)
    acc_hh = np.zeros((oh, ow), np.float32)
    acc_x = np.zeros((oh, ow), np.float32)

    def instruction(acc, a, b, rows):
        blk = np.zeros((oh, ow), np.float64)                  # the sum inside one instruction is taken as exact
        for p in rows:
            for q in range(kw):
                blk += a[p, q] * b[p:p + oh, q:q + ow]
        return (acc.astype(np.float64) + blk).astype(np.float32)

    for g0 in range(-(phase % 2), kh, 2):
        rows = [p for p in (g0, g0 + 1) if 0 <= p < kh]
        if "lh" in products:
            acc_x = instruction(acc_x, fl, xh, rows)
        if "hh" in products:
            acc_hh = instruction(acc_hh, fh, xh, rows)
        if "hl" in products:
            acc_x = instruction(acc_x, fh, xl, rows)
    inv = np.float32(1.0 / (ts * X_SCALE))
    y = acc_x * np.float32(inv / np.float32(lo_scale)) + acc_hh * inv     # fp32, as the kernel's last two instructions
    return y.astype(np.float64)


def _case(shape, kshape, x_range=(0.0, 1.0)):
    wl = W.WORKLOADS["conv2d_8k_11x11"]
    x, f = W.make(wl, x_shape=shape)
    if kshape != f.shape:
        f = np.ascontiguousarray(f[:kshape[0], :kshape[1]])
    lo, hi = x_range
    x = (x * np.float32(hi - lo) + np.float32(lo)).astype(np.float32)
    return x, f


@pytest.mark.parametrize("phase", [0, 1])
def test_split_fp16_three_products_meet_the_bound_with_margin(phase):
    x, f = _case((200, 300), (11, 11))
    ref, scale = oracle.conv2d(x, f), oracle.absdot2d(x, f)
    e = oracle.max_rel_err(_model(x, f, phase=phase), ref, scale)
    assert e <= 3e-6 / 3, f"split-fp16 model: {e}"            # measured 5e-8: a margin of 200 under 1e-5


def test_signed_data_and_other_filter_sizes():
    for kshape, x_range in (((3, 3), (-1.0, 1.0)), ((5, 5), (-7.9, 7.9)), ((13, 13), (0.0, 1.0)), ((1, 13), (-1.0, 1.0))):
        x, f = _case((120, 200), kshape, x_range)
        ref, scale = oracle.conv2d(x, f), oracle.absdot2d(x, f)
        e = oracle.max_rel_err(_model(x, f), ref, scale)
        assert e <= 1e-6, f"{kshape} on {x_range}: {e}"


def test_the_cross_terms_are_needed():
    x, f = _case((120, 200), (11, 11))
    ref, scale = oracle.conv2d(x, f), oracle.absdot2d(x, f)
    assert oracle.max_rel_err(_model(x, f, products=("hh",)), ref, scale) > 1e-5          # fp16 alone: 1.1e-4
    assert oracle.max_rel_err(_model(x, f, products=("hh", "lh")), ref, scale) > 1e-5     # inputs unsplit: 9e-5


def test_small_inputs_need_the_enlarged_lo_parts():
    # Inputs in [2^-17, 2^-16]: times 2^13 they are normal fp16 numbers, but their remainders (2^-11 of that) are not.
    x, f = _case((60, 90), (5, 5), x_range=(0.5, 1.0))
    x = (x * np.float32(2.0 ** -16)).astype(np.float32)
    ref, scale = oracle.conv2d(x, f), oracle.absdot2d(x, f)
    assert oracle.max_rel_err(_model(x, f), ref, scale) <= 1e-6
    assert oracle.max_rel_err(_model(x, f, lo_scale=1.0), ref, scale) > 1e-5


def test_inputs_below_2_to_the_minus_27_count_as_zero():
    x, f = _case((40, 60), (3, 3))
    tiny = (x * np.float32(2.0 ** -29)).astype(np.float32)     # < 2^-28: hi is an fp16 subnormal, read as zero
    assert np.all(_model(tiny, f) == 0.0)
