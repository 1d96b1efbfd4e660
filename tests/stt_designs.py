"""Designs used by the tests of the generic space-time-transform path: (alloc, sched, dep_x, dep_w, dep_z)."""
from paper_2010_15884_amd import schedule_model as sm


def named(d):
    t, e = sm.TRANSFORMS[d], sm.DEPENDENCES[d]
    return t.alloc, t.sched, e.get("X"), e.get("W"), e["Z"]


PAPER = {d: named(d) for d in sm.TRANSFORMS}

# valid designs that are not in the paper's tables
NOVEL = {
    "BBS": ((1, 0), (1, 1), None, None, (0, 1)),                 # everything loaded, sums stay, skewed start
    "SBM_half_speed": ((1, 1), (1, 2), (-1, 1), None, (0, 1)),   # sums move every second step
    "FBS_mirrored": ((-1, 0), (0, 1), (-1, 1), None, (0, 1)),    # PE index runs against c
    "FSM_mirrored": ((0, -1), (1, -1), (1, -1), (1, 0), (0, -1)),
    "FBS_descending": ((1, 0), (0, -1), (1, -1), None, (0, -1)),  # taps taken from the last to the first
}

# designs Section 2.2 rules out, with the reason
INVALID = {
    "singular": ((1, 1), (1, 1), None, None, (0, 1)),                      # det = 0
    "sums_read_before_they_exist": ((1, 0), (1, 0), None, None, (0, 1)),   # s.ez = 0 (and singular)
    "sbm_run_backwards": ((1, 1), (0, -1), (-1, 1), None, (0, 1)),         # s.ez = -1
    "fbs_inputs_from_the_future": ((1, 0), (0, 1), (1, -1), None, (0, 1)),  # s.ex = -1
    "bfs_weights_same_step": ((1, 0), (0, 1), None, (1, 0), (0, 1)),       # s.ew = 0
    "x_dependence_changes_the_input": ((1, 0), (0, 1), (-1, 2), None, (0, 1)),
    "x_dependence_null": ((1, 0), (0, 1), (0, 0), None, (0, 1)),
    "w_dependence_changes_the_tap": ((1, 0), (1, 1), None, (1, 1), (0, 1)),
    "z_dependence_across_outputs": ((1, 0), (1, 1), None, None, (1, 1)),
    "z_dependence_skips_taps": ((1, 0), (0, 1), None, None, (0, 2)),
}

# valid designs this kernel is not built for
TOO_LARGE = {
    "det_2": ((1, 0), (1, 2), None, None, (0, 1)),                         # holes in the PE-time grid
    "values_jump_over_pes": ((1, 3), (0, 1), (-1, 1), None, (0, 1)),       # P.ex = 2, P.ez = 3
    "weights_travel_four_steps": ((1, 0), (4, 1), None, (1, 0), (0, 1)),   # s.ew = 4
    "huge_coefficient": ((65, 1), (64, 1), None, None, (0, 1)),
}
