"""The oracle against the paper's own recurrence equations and schedules.

The six 1-D designs (Section 3.1, Table 2) and the 2-D SBM design (Section 5)
all define the same function as Eq. 2 / Eq. 3.  Evaluated literally in fp64 on
small sizes they must reproduce the oracle; run under their space-time
transforms they must still do so, and use the numbers of lanes and steps that
Table 4 is computed from.
"""
import os

import numpy as np
import pytest

import oracle
from paper_2010_15884_amd import schedule_model as sm
from ure_designs import systolic_1d, systolic_2d_sbm, ure_1d, ure_2d_sbm

DESIGNS = ["SBM", "BSM", "FSM", "BFS", "FFS", "FBS"]
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _ints(seed, n, k):
    rng = np.random.default_rng(seed)
    return (rng.integers(-9, 10, n).astype(np.float32), rng.integers(-5, 6, k).astype(np.float32))


@pytest.mark.parametrize("design", DESIGNS)
@pytest.mark.parametrize("n,k", [(20, 5), (16, 16), (9, 1), (13, 2), (40, 7)])
def test_recurrences_equal_the_definition(design, n, k):
    x, w = _ints(n * 31 + k, n, k)
    assert np.array_equal(ure_1d(design, x, w), oracle.conv1d(x, w))


@pytest.mark.parametrize("design", DESIGNS)
def test_recurrences_on_random_floats(design):
    rng = np.random.default_rng(5)
    x = rng.uniform(-1, 1, 64).astype(np.float32)
    w = rng.uniform(-1, 1, 16).astype(np.float32)
    assert np.allclose(ure_1d(design, x, w), oracle.conv1d(x, w), rtol=0, atol=1e-14)


def test_stride2_fbs_recurrence_reading():
    # Table 2's stride-2 cell hands X on two taps later; that is consistent only
    # with Z(c) = sum_q x(2c+q) w(q), i.e. every second output of the stride-1 result.
    x, w = _ints(77, 41, 5)
    full = oracle.conv1d(x, w)
    assert np.array_equal(ure_1d("FBS", x, w, stride=2), full[::2])
    for n, k in [(41, 5), (40, 5), (30, 2), (37, 16), (19, 1)]:
        x, w = _ints(n * 10 + k, n, k)
        assert np.array_equal(ure_1d("FBS", x, w, stride=2), oracle.conv1d_strided(x, w, 2))


@pytest.mark.parametrize("shape,kshape", [((6, 9), (2, 2)), ((8, 12), (5, 5)), ((5, 7), (3, 1)), ((4, 11), (1, 4)), ((9, 9), (3, 5))])
def test_2d_sbm_recurrence_and_schedule(shape, kshape):
    rng = np.random.default_rng(shape[0] * 100 + kshape[1])
    x = rng.integers(-9, 10, shape).astype(np.float32)
    f = rng.integers(-5, 6, kshape).astype(np.float32)
    want = oracle.conv2d(x, f)
    assert np.array_equal(ure_2d_sbm(x, f), want)
    got, n_pe, steps = systolic_2d_sbm(x, f)
    assert np.array_equal(got, want)
    assert n_pe == want.shape[1] + kshape[1] - 1          # PE = c + q
    assert steps == kshape[0] * kshape[1]                  # t = p + P q


@pytest.mark.parametrize("design", DESIGNS)
@pytest.mark.parametrize("n_out,k", [(16, 5), (16, 2), (7, 3), (64, 16)])
def test_transformed_schedule_computes_the_definition(design, n_out, k):
    x, w = _ints(n_out + 17 * k, n_out + k - 1, k)
    t = sm.TRANSFORMS[design]
    got, lanes, steps = systolic_1d(design, (t.alloc, t.sched), x, w)
    assert np.array_equal(got, oracle.conv1d(x, w))
    m = sm.model(design, n_out, k)
    assert (lanes, steps) == (m["lanes"], m["steps"])


@pytest.mark.parametrize("design", DESIGNS)
def test_validity_conditions(design):
    assert sm.is_valid(design)
    assert sm.DEPENDENCES[design] == __import__("ure_designs")._DEPS[design]


def test_an_invalid_transform_is_rejected_by_the_simulator():
    # BFS equations with FBS's transform: the forwarded weight would have to
    # arrive in the same step it is produced (s^T e = 0).
    x, w = _ints(3, 20, 5)
    with pytest.raises(AssertionError):
        systolic_1d("BFS", ((1, 0), (0, 1)), x, w)


def test_naming_matches_data_movement():
    # (input, weight, psum): Stay = space distance 0, Forwarded / Migrated = +-1 PE.
    mv = {d: sm.movement(d) for d in DESIGNS}
    assert mv["SBM"]["X"][0] == 0 and mv["SBM"]["Z"][0] == 1        # inputs Stay, psums Migrate
    assert mv["FBS"]["X"][0] == -1 and mv["FBS"]["Z"][0] == 0       # inputs Forwarded, psums Sediment
    assert mv["BSM"]["W"][0] == 0 and mv["BSM"]["Z"][0] == 1        # weights Stay, psums Migrate
    assert mv["FSM"]["X"][0] == -1 and mv["FSM"]["W"][0] == 0 and mv["FSM"]["Z"][0] == -1
    assert mv["BFS"]["W"][0] == 1 and mv["BFS"]["Z"][0] == 0        # weights Forwarded, psums Sediment
    assert mv["FFS"]["X"][0] == 1 and mv["FFS"]["W"][0] == 1 and mv["FFS"]["Z"][0] == 0
    for d in DESIGNS:
        for _, (_, dt) in mv[d].items():
            assert dt >= 1


def test_table4_printed_values():
    rows = {}
    with open(os.path.join(GOLDEN, "table4_model.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            name, outturn, util, regs = line.split()
            rows[name] = (float(outturn), float(util), int(regs))
    assert set(rows) == set(DESIGNS)
    for name, (outturn, util, regs) in rows.items():
        m = sm.model(name, 16, 5)
        assert m["registers"] == regs, name
        # the paper prints two significant digits
        assert abs(m["outturn"] - outturn) < 0.005 + 1e-12, name
        assert abs(100 * m["utilisation"] - util) < 0.5, name
    # the (lanes, steps) pairs behind the table
    assert {d: (sm.model(d)["lanes"], sm.model(d)["steps"]) for d in DESIGNS} == {
        "SBM": (20, 5), "BSM": (5, 20), "FSM": (5, 20), "BFS": (16, 20), "FFS": (16, 35), "FBS": (16, 5)}


def test_sbm_vector_length_is_q_plus_ccc_minus_1():
    # Section 3.1: the compiler sizes the SBM register vectors as Q + CCC - 1.
    for ccc, q in [(16, 5), (64, 16), (8, 2)]:
        assert sm.model("SBM", ccc, q)["lanes"] == q + ccc - 1


def test_wave64_model():
    fbs = sm.wave64("FBS", 16)
    assert fbs["utilisation"] == 1.0 and fbs["steps"] == 16
    sbm = sm.wave64("SBM", 16)
    assert sbm["utilisation"] == pytest.approx((1024 - 15) / 1024)
    # K-lane arrays: 12 arrays of 5 lanes, segments of 84 outputs, 88 steps
    bsm = sm.wave64("BSM", 5)
    assert (bsm["steps"], bsm["outturn"]) == (88, pytest.approx(12 * 84 / 88))
    assert bsm["utilisation"] == pytest.approx(12 * 84 * 5 / (64 * 88))
    assert sm.wave64("FSM", 5) == bsm
    # FFS with 16-PE arrays has exactly the paper's Table 4 utilisation at K = 5: 16*5/(16*35)
    assert sm.wave64("FFS", 5)["utilisation"] == pytest.approx(sm.model("FFS", 16, 5)["utilisation"])
    assert sm.wave64("BFS", 5)["utilisation"] == pytest.approx(5 / 8)


def test_model_of_unlisted_designs():
    # SBM whose sums move every second step: PE = c + q, time = c + 2q -> 20 lanes, 24 steps for 16 outputs, 5 taps
    m = sm.model_of(sm.Transform((1, 1), (1, 2)), {"X": (-1, 1), "Z": (0, 1)}, 16, 5)
    assert (m["lanes"], m["steps"]) == (20, 24)
    assert m["utilisation"] == pytest.approx(80 / (20 * 24))
    assert m["registers"] == 16 * (2 + 1 + 3)                    # X waits one step, W is loaded, Z two steps
    # everything loaded, sums stay, skewed start: the BFS schedule without weight forwarding
    m = sm.model_of(sm.Transform((1, 0), (1, 1)), {"Z": (0, 1)}, 16, 5)
    assert (m["lanes"], m["steps"], m["registers"]) == (16, 20, 16 * 4)
