"""CPU models of the lane programs the tap-array kernels run (test helper).

Each function executes, step by step on numpy vectors of 64 "lanes", exactly the
register moves / selects / multiply-adds that the BSM, FSM and FFS kernels issue
per time step (paper Table 2), for ONE wavefront.  They exist to pin the lane
logic -- shift directions, boundary selects, the time at which a PE's result is
complete -- on the CPU before and beside the GPU run.  They share no code with the
oracle (and none with the kernels: this is Python).
"""
import numpy as np

LANES = 64


def _below(v, fill=0.0):
    """lane l takes lane l-1 (DPP wave_shr:1); lane 0 takes `fill`."""
    out = np.empty_like(v)
    out[1:] = v[:-1]
    out[0] = fill
    return out


def _above(v, fill=0.0):
    """lane l takes lane l+1 (DPP wave_shl:1); lane 63 takes `fill`."""
    out = np.empty_like(v)
    out[:-1] = v[1:]
    out[-1] = fill
    return out


def bsm_wave(x, w, seg):
    """BSM (Table 2, row 1 left): PE = tap q, time = c + q.  Weights stay, the input
    x(t) is broadcast to the K PEs of an array, partial sums move one PE up per step.
    A wavefront holds A = 64 // K arrays; array a produces outputs [a*seg, (a+1)*seg)."""
    x = np.asarray(x, np.float64)
    k = len(w)
    arrays = LANES // k
    lane = np.arange(LANES)
    a, q = lane // k, lane % k
    active = a < arrays
    wq = np.where(active, np.asarray(w, np.float64)[q], 0.0)
    z = np.zeros(LANES)
    y = np.full(arrays * seg, np.nan)
    for t in range(seg + k - 1):
        xin = x[np.minimum(a * seg + t, len(x) - 1)]          # same address for the K lanes of an array
        zprev = np.where(q == 0, 0.0, _below(z))
        z = zprev + xin * wq
        c = t - (k - 1)
        if 0 <= c < seg:
            for arr in range(arrays):                           # lanes with q == K-1 store
                y[arr * seg + c] = z[arr * k + k - 1]
    return y


def fsm_wave(x, w, seg):
    """FSM (Table 2, row 1 right): PE = tap q, time = c - q.  Weights stay; inputs move
    towards lower q at half speed (two steps per PE); partial sums move towards lower q,
    start at PE K-1 and leave at PE 0."""
    x = np.asarray(x, np.float64)
    k = len(w)
    arrays = LANES // k
    lane = np.arange(LANES)
    a, q = lane // k, lane % k
    active = a < arrays
    wq = np.where(active, np.asarray(w, np.float64)[q], 0.0)
    z = np.zeros(LANES)
    x1 = np.zeros(LANES)                                        # X computed one step ago
    x2 = np.zeros(LANES)                                        # X computed two steps ago
    y = np.full(arrays * seg, np.nan)
    for t in range(-(k - 1), seg):
        c = t + q                                               # output this PE works on
        idx = np.clip(t + 2 * q, 0, seg + k - 2)               # c + q, clamped into the array's window
        xload = x[np.minimum(a * seg + idx, len(x) - 1)]
        xt = np.where((q == k - 1) | (c == 0), xload, _above(x2))
        zprev = np.where(q == k - 1, 0.0, _above(z))
        z = zprev + xt * wq
        x2, x1 = x1, xt
        if 0 <= t < seg:
            for arr in range(arrays):                           # lanes with q == 0 store output t
                y[arr * seg + t] = z[arr * k]
    return y


def ffs_wave(x, w, width=16):
    """FFS (Table 2, row 2 right): PE = output c, time = 2c + q.  Inputs move up one PE
    per step, weights move up one PE per two steps, partial sums stay.  A wavefront holds
    64 // width arrays of `width` PEs; array a produces outputs [a*width, (a+1)*width)."""
    x = np.asarray(x, np.float64)
    k = len(w)
    arrays = LANES // width
    lane = np.arange(LANES)
    a, c = lane // width, lane % width
    z = np.zeros(LANES)
    xt = np.zeros(LANES)
    w1 = np.zeros(LANES)
    w2 = np.zeros(LANES)
    wpad = np.concatenate([np.asarray(w, np.float64), np.zeros(2 * width)])
    for t in range(2 * (width - 1) + k):
        q = t - 2 * c
        valid = (q >= 0) & (q < k)
        idx = np.clip(t - c, 0, width + k - 2)                  # c + q = t - c
        xload = x[np.minimum(a * width + idx, len(x) - 1)]
        xt = np.where((c == 0) | (q == k - 1), xload, _below(xt))
        wt = np.where(c == 0, wpad[min(t, len(wpad) - 1)], _below(w2))
        z = np.where(valid, z + xt * wt, z)
        w2, w1 = w1, wt
    return z[: arrays * width]


# ------------------------------------------------------------------ generic space-time transform
def stt_plan(alloc, sched, dep_x, dep_w, dep_z, k, lanes=LANES):
    """Host-side bookkeeping of the generic kernel for one wavefront: outputs per chunk C, the lowest
    PE and time coordinates, the number of steps, and (lane distance, time distance) per variable.
    Mirrors Section 2.2 / Section 4.1: PE = P.z, time = s.z, a value passed along e travels P.e PEs
    in s.e steps."""
    p0, p1 = alloc
    s0, s1 = sched
    det = p0 * s1 - p1 * s0
    assert det in (1, -1)
    C = lanes if p0 == 0 else (lanes - 1 - abs(p1) * (k - 1)) // abs(p0) + 1
    C = min(C, lanes)
    assert C >= 1
    pmin = min(0, p0 * (C - 1)) + min(0, p1 * (k - 1))
    tmin = min(0, s0 * (C - 1)) + min(0, s1 * (k - 1))
    steps = abs(s0) * (C - 1) + abs(s1) * (k - 1) + 1
    dist = {}
    for name, e in (("X", dep_x), ("W", dep_w), ("Z", dep_z)):
        dist[name] = None if e is None else (p0 * e[0] + p1 * e[1], s0 * e[0] + s1 * e[1])
    return dict(det=det, C=C, pmin=pmin, tmin=tmin, steps=steps, dist=dist)


def stt_wave(alloc, sched, dep_x, dep_w, dep_z, x, w, lanes=LANES):
    """One wavefront of the generic kernel: every lane is a PE; per time step each lane inverts the
    transform to find its iteration point (c, q), takes X / W / Z either from memory (no dependence, or
    the producer z - e lies outside the chunk) or from its neighbour's history, and multiplies-adds.
    Returns the outputs of the first chunk (min(C, len(x)-k+1) of them)."""
    x = np.asarray(x, np.float64)
    w = np.asarray(w, np.float64)
    k = len(w)
    pl = stt_plan(alloc, sched, dep_x, dep_w, dep_z, k, lanes)
    p0, p1 = alloc
    s0, s1 = sched
    det, C = pl["det"], pl["C"]
    Cv = min(C, len(x) - k + 1)                                  # outputs that exist in this chunk
    lane = np.arange(lanes)
    hist = {v: [np.zeros(lanes) for _ in range(3)] for v in "XWZ"}
    y = np.full(Cv, np.nan)

    def moved(var):
        dl, dt = pl["dist"][var]
        v = hist[var][dt - 1]                                    # produced dt steps ago ...
        if dl == 1:
            return _below(v)                                     # ... by the PE one below
        if dl == -1:
            return _above(v)
        return v

    for t in range(pl["steps"]):
        pp, tp = lane + pl["pmin"], t + pl["tmin"]
        c = det * (s1 * pp - p1 * tp)
        q = det * (-s0 * pp + p0 * tp)
        valid = (c >= 0) & (c < Cv) & (q >= 0) & (q < k)
        xin = x[np.clip(c + q, 0, len(x) - 1)]
        win = w[np.clip(q, 0, k - 1)]

        def inside(e):
            cc, qq = c - e[0], q - e[1]
            return (cc >= 0) & (cc < Cv) & (qq >= 0) & (qq < k)

        xv = xin if dep_x is None else np.where(inside(dep_x), moved("X"), xin)
        wv = win if dep_w is None else np.where(inside(dep_w), moved("W"), win)
        zv = np.where(inside(dep_z), moved("Z"), 0.0) + xv * wv
        last = valid & ~(((q + dep_z[1]) >= 0) & ((q + dep_z[1]) < k))
        for l in np.nonzero(last)[0]:
            y[c[l]] = zv[l]
        for var, val in (("X", xv), ("W", wv), ("Z", zv)):
            hist[var] = [val, hist[var][0], hist[var][1]]
    return y
