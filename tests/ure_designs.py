"""Test helpers: the paper's recurrence equations, evaluated literally.

``ure_1d(design, x, w)`` fills the tables X, W, Z over the (c, q) iteration
space exactly as the uniform recurrence equations of Section 3.1 (SBM / FBS)
and Table 2 (BSM, FSM, BFS, FFS, FBS stride 2) state them, in fp64.
``ure_2d_sbm`` does the same for the four-index equations of Section 5.

``systolic_1d`` executes a design after its space-time transform (Section 2.2,
Section 4.1): time step by time step, every PE computes the iteration point the
inverse transform gives it and may only read values that a PE produced at an
EARLIER step (or the same step for nothing at all).  It returns the outputs and
the number of PEs and time steps really used.

None of this is shared with the oracle or the GPU path.
"""
from functools import lru_cache

import numpy as np


def ure_1d(design, x, w, stride=1):
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    Q = len(w)
    C = (len(x) - Q) // stride + 1

    @lru_cache(maxsize=None)
    def X(c, q):
        if design in ("SBM", "FBS"):
            if stride == 1:
                return x[c + q] if (q == 0 or c == C - 1) else X(c + 1, q - 1)
            # stride-2 FBS of Table 2: an input is handed on two taps later.
            # The printed x(c+q) cannot be meant together with X(c+1, q-2);
            # the definition must read x(stride*c + q).
            return x[stride * c + q] if (q < stride or c == C - 1) else X(c + 1, q - stride)
        if design in ("BSM", "BFS"):
            return x[c + q]
        if design in ("FSM", "FFS"):
            return x[c + q] if (c == 0 or q == Q - 1) else X(c - 1, q + 1)
        raise KeyError(design)

    @lru_cache(maxsize=None)
    def W(c, q):
        if design in ("SBM", "FBS"):
            return w[q]
        return w[q] if c == 0 else W(c - 1, q)

    @lru_cache(maxsize=None)
    def Z(c, q):
        if design == "FSM":                                 # accumulates with q descending
            prev = 0.0 if q == Q - 1 else Z(c, q + 1)
        else:
            prev = 0.0 if q == 0 else Z(c, q - 1)
        return prev + X(c, q) * W(c, q)

    last = 0 if design == "FSM" else Q - 1
    return np.array([Z(c, last) for c in range(C)])


def ure_2d_sbm(x, f):
    """Section 5 equations.  x[r][c] row-major, f[p][q]; the paper writes
    x(c+q, r+p) and w(q, p) with c, q the systolic axis."""
    x = np.asarray(x, dtype=np.float64)
    f = np.asarray(f, dtype=np.float64)
    P, Q = f.shape
    R, C = x.shape[0] - P + 1, x.shape[1] - Q + 1

    @lru_cache(maxsize=None)
    def X(c, p, q, r):
        return x[r + p, c + q] if (c == C - 1 or q == 0) else X(c + 1, p, q - 1, r)

    @lru_cache(maxsize=None)
    def Z(c, p, q, r):
        if p == 0 and q == 0:
            prev = 0.0
        elif p == 0:
            prev = Z(c, P - 1, q - 1, r)
        else:
            prev = Z(c, p - 1, q, r)
        return prev + X(c, p, q, r) * f[p, q]

    return np.array([[Z(c, P - 1, Q - 1, r) for c in range(C)] for r in range(R)])


# dependence vectors: variable at z = (c, q) reads itself at z - e
_DEPS = {
    "SBM": {"X": (-1, 1), "Z": (0, 1)},
    "FBS": {"X": (-1, 1), "Z": (0, 1)},
    "BSM": {"W": (1, 0), "Z": (0, 1)},
    "BFS": {"W": (1, 0), "Z": (0, 1)},
    "FSM": {"X": (1, -1), "W": (1, 0), "Z": (0, -1)},
    "FFS": {"X": (1, -1), "W": (1, 0), "Z": (0, 1)},
}


def systolic_1d(design, transform, x, w):
    """Run ``design`` under ``transform`` = ((Pc, Pq), (sc, sq)).

    Register files are modelled as values tagged with the (PE, time) that
    produced them; a read of V(z - e) must find a value produced at PE
    pe - P.e at time t - s^T e, with s^T e >= 1.
    """
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    Q = len(w)
    C = len(x) - Q + 1
    (pc, pq), (sc, sq) = transform
    det = pc * sq - pq * sc
    assert det in (1, -1), "all six designs have unimodular transforms"
    pts = {}
    for c in range(C):
        for q in range(Q):
            key = (pc * c + pq * q, sc * c + sq * q)
            assert key not in pts, "two iteration points on one PE at one time"
            pts[key] = (c, q)
    pes = sorted({k[0] for k in pts})
    times = sorted({k[1] for k in pts})
    regs = {"X": {}, "W": {}, "Z": {}}
    deps = _DEPS[design]
    out = np.zeros(C)

    def passed(var, pe, t):
        e = deps[var]
        dist_s = pc * e[0] + pq * e[1]
        dist_t = sc * e[0] + sq * e[1]
        assert dist_t >= 1, f"{design}: {var} would be read before it exists"
        return regs[var][(pe - dist_s, t - dist_t)]

    for t in range(times[0], times[-1] + 1):
        for pe in pes:
            if (pe, t) not in pts:
                continue                                    # PE idle at this step
            c, q = pts[(pe, t)]
            # X
            if design in ("SBM", "FBS"):
                xv = x[c + q] if (q == 0 or c == C - 1) else passed("X", pe, t)
            elif design in ("BSM", "BFS"):
                xv = x[c + q]
            else:
                xv = x[c + q] if (c == 0 or q == Q - 1) else passed("X", pe, t)
            # W
            if design in ("SBM", "FBS"):
                wv = w[q]
            else:
                wv = w[q] if c == 0 else passed("W", pe, t)
            # Z
            if design == "FSM":
                zprev = 0.0 if q == Q - 1 else passed("Z", pe, t)
                done = q == 0
            else:
                zprev = 0.0 if q == 0 else passed("Z", pe, t)
                done = q == Q - 1
            zv = zprev + xv * wv
            regs["X"][(pe, t)] = xv
            regs["W"][(pe, t)] = wv
            regs["Z"][(pe, t)] = zv
            if done:
                out[c] = zv
    return out, len(pes), times[-1] - times[0] + 1


def systolic_2d_sbm(x, f):
    """Section 5 / Fig. 5 design: for every row r, PE = c + q, time = p + P*q."""
    x = np.asarray(x, dtype=np.float64)
    f = np.asarray(f, dtype=np.float64)
    P, Q = f.shape
    R, C = x.shape[0] - P + 1, x.shape[1] - Q + 1
    out = np.zeros((R, C))
    n_pe = C + Q - 1
    for r in range(R):
        zreg = {}
        xreg = {}
        for t in range(P * Q):
            q, p = divmod(t, P)
            for pe in range(n_pe):
                c = pe - q
                if not (0 <= c < C):
                    continue
                # inputs stay: X(c,p,q) = X(c+1,p,q-1) lives on the same PE, P steps earlier
                if c == C - 1 or q == 0:
                    xv = x[r + p, c + q]
                else:
                    xv = xreg[(pe, t - P)]
                if p == 0 and q == 0:
                    zprev = 0.0
                elif p == 0:
                    zprev = zreg[(pe - 1, t - 1)]           # partial sum migrates one PE
                else:
                    zprev = zreg[(pe, t - 1)]               # and rests while p advances
                zv = zprev + xv * f[p, q]
                xreg[(pe, t)] = xv
                zreg[(pe, t)] = zv
                if p == P - 1 and q == Q - 1:
                    out[r, c] = zv
    return out, n_pe, P * Q
