"""Space-time transforms of the paper's systolic designs and its analytical model.

A design maps an iteration point (c, q) -- output position c, tap q -- to a
processing element P.z and a time step s^T.z (paper Section 2.2).  The table
below restates the transforms of Section 3.1 (SBM) and Table 2 (the other
five), and ``model`` evaluates the paper's Section 6.2 model:

    outturn     = outputs / #time steps
    utilisation = outputs * taps / (#lanes * #time steps)

where #lanes is the length of the *virtual* PE vector (the extent of P.z) and
#time steps the extent of s^T.z, and the table's register count: every variable
keeps one value per PE, a passed variable s^T.e more (the history of Section
4.1's general code), over 16 PEs for the designs that give each output its own
PE (SBM counted with its 16 outputs, not its 20 vector lanes) and over Q PEs
for those whose PE is the tap.  With 16 outputs and 5 taps this reproduces all
eighteen numbers of the paper's Table 4.

``wave64`` evaluates the same two figures for the way the HIP kernels lay each
design over a 64-lane wavefront.

Host-side bookkeeping only: no convolution arithmetic lives here.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple


@dataclass(frozen=True)
class Transform:
    """Rows of the 2x2 transform matrix over (c, q): allocation P and schedule s."""
    alloc: Tuple[int, int]
    sched: Tuple[int, int]

    @property
    def det(self) -> int:
        return self.alloc[0] * self.sched[1] - self.alloc[1] * self.sched[0]


# (input, weight, partial sum) naming of Section 3.1: Broadcast / Forwarded / Stay,
# Migrated / Sedimented.
TRANSFORMS: Dict[str, Transform] = {
    "SBM": Transform((1, 1), (0, 1)),    # s = c + q, t = q        (Section 3.1)
    "BSM": Transform((0, 1), (1, 1)),    # s = q,     t = c + q    (Table 2, row 1 left)
    "FSM": Transform((0, 1), (1, -1)),   # s = q,     t = c - q    (Table 2, row 1 right)
    "BFS": Transform((1, 0), (1, 1)),    # s = c,     t = c + q    (Table 2, row 2 left)
    "FFS": Transform((1, 0), (2, 1)),    # s = c,     t = 2c + q   (Table 2, row 2 right)
    "FBS": Transform((1, 0), (0, 1)),    # s = c,     t = q        (Table 2, row 3 left)
}

# Dependence vectors e (a variable at z reads its value from z - e), per design.
# None = the variable is loaded / broadcast, not passed between iterations.
DEPENDENCES: Dict[str, Dict[str, Tuple[int, int]]] = {
    "SBM": {"X": (-1, 1), "Z": (0, 1)},
    "FBS": {"X": (-1, 1), "Z": (0, 1)},
    "BSM": {"W": (1, 0), "Z": (0, 1)},
    "BFS": {"W": (1, 0), "Z": (0, 1)},
    "FSM": {"X": (1, -1), "W": (1, 0), "Z": (0, -1)},
    "FFS": {"X": (1, -1), "W": (1, 0), "Z": (0, 1)},
}


def extent(row: Tuple[int, int], n_out: int, n_taps: int) -> int:
    """Number of distinct values of row.(c, q) over 0<=c<n_out, 0<=q<n_taps."""
    return abs(row[0]) * (n_out - 1) + abs(row[1]) * (n_taps - 1) + 1


def is_valid(design: str) -> bool:
    """Section 2.2: every dependence needs s^T e >= 0 and != 0 (none of the
    passed variables is a broadcast); two points on one PE must differ in
    time, i.e. the transform must not be singular."""
    t = TRANSFORMS[design]
    if t.det == 0:
        return False
    for e in DEPENDENCES[design].values():
        if t.sched[0] * e[0] + t.sched[1] * e[1] <= 0:
            return False
    return True


def movement(design: str) -> Dict[str, Tuple[int, int]]:
    """(space distance P.e, time distance s^T e) of every passed variable."""
    t = TRANSFORMS[design]
    return {v: (t.alloc[0] * e[0] + t.alloc[1] * e[1], t.sched[0] * e[0] + t.sched[1] * e[1])
            for v, e in DEPENDENCES[design].items()}


def model_of(transform: Transform, deps: Dict[str, Tuple[int, int]], n_out: int = 16, n_taps: int = 5) -> Dict[str, float]:
    """Section 6.2's figures for any design given as a transform and the dependence
    vectors of its passed variables (a subset of X, W, Z)."""
    lanes = extent(transform.alloc, n_out, n_taps)
    steps = extent(transform.sched, n_out, n_taps)
    depth = sum((transform.sched[0] * deps[v][0] + transform.sched[1] * deps[v][1] + 1) if v in deps else 1
                for v in "XWZ")
    pes = n_out if transform.alloc[0] != 0 else n_taps
    return {
        "lanes": lanes,
        "steps": steps,
        "outturn": n_out / steps,
        "utilisation": n_out * n_taps / (lanes * steps),
        "registers": pes * depth,
    }


def model(design: str, n_out: int = 16, n_taps: int = 5) -> Dict[str, float]:
    """The same for one of the paper's six designs."""
    return model_of(TRANSFORMS[design], DEPENDENCES[design], n_out, n_taps)


def wave64(design: str, n_taps: int, groups: int = 4, tile: int = 4, lanes: int = 64) -> Dict[str, float]:
    """The same model for the way the HIP kernels lay each design over a 64-lane
    wavefront.  "lanes" counts PE slots, "steps" time steps, utilisation is the share
    of PE-steps that are useful multiply-adds.

    FBS: a wavefront streams ``groups`` register groups of ``lanes`` x ``tile`` PEs; every
         PE owns one output and runs n_taps steps, all useful.
    SBM: the PE vector also carries the n_taps-1 slots the partial sums migrate through,
         so a chunk yields n_taps-1 fewer outputs (the paper's vector length Q+CCC-1).
    BFS: every lane is a ``tile``-PE array; an array sees n_taps+tile-1 inputs, and a PE
         is busy for n_taps of them (idle PE-steps are not issued on the GPU: the PEs of
         a lane share one ALU).
    BSM, FSM: arrays are n_taps lanes long, lanes // n_taps of them per wavefront, each
         streaming a segment of ~1024 / arrays outputs with one fill / drain of n_taps-1.
    FFS: arrays of 16 PEs (the paper's size), 2*15 + n_taps steps for 16 outputs each.
    """
    if design in ("FBS", "SBM"):
        n_pe = lanes * tile * groups
        outs = n_pe if design == "FBS" else n_pe - (n_taps - 1)
        steps = n_taps
    elif design == "BFS":
        n_pe = lanes * tile * groups
        outs, steps = n_pe, n_taps + tile - 1
    elif design in ("BSM", "FSM"):
        arrays = lanes // n_taps
        seg = (((1024 // arrays) - 4) & ~7) + 4
        n_pe, outs, steps = lanes, arrays * seg, seg + n_taps - 1
    elif design == "FFS":
        width = 16
        n_pe, outs, steps = lanes, lanes, 2 * (width - 1) + n_taps
    else:
        raise ValueError(design)
    return {"lanes": n_pe, "steps": steps, "outturn": outs / steps,
            "utilisation": outs * n_taps / (n_pe * steps)}
