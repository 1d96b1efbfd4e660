"""SYS_PROJ_AUTO is a measured choice: on each of the five benchmark workloads, and on two images whose pitch is not
a power of two (where the rule differs), it must be as fast as the fastest projection the library has built for that
filter (the opt-in matrix-core projection aside, which AUTO never picks because it restricts the input range).

Timing method: batches of back-to-back launches on rotated buffers (past the 256 MB memory-side cache) between two
events, best of five batches per projection, projections interleaved so that clock and thermal drift hit all of
them alike.  The two small workloads are bound by the host's launch path when launched one by one (7 - 8 us per
call whatever the kernel), so their launches are replayed from a HIP graph, 100 per replay, which leaves the
kernels' own time.  Tolerance 5 %: repeated runs of one kernel on one box differ by 2 - 3 %.
"""
import pytest
import torch

from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import workloads as W

pytestmark = pytest.mark.gpu

TOLERANCE = 1.05


def _batch_time(fn, launches):
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for i in range(launches):
        fn(i)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / launches


_BASE = W.WORKLOADS["conv2d_4k_5x5"]
EXTRA = {   # away from the benchmark sizes: 20 KB and 24 KB pitches
    "conv2d_5120_5x5": W.Workload("conv2d_5120_5x5", 2, (5120, 5120), (5, 5), _BASE.x_range, _BASE.w_range, _BASE.seed + 11),
    "conv2d_6144_7x7": W.Workload("conv2d_6144_7x7", 2, (6144, 6144), (7, 7), _BASE.x_range, _BASE.w_range, _BASE.seed + 12),
}


@pytest.mark.parametrize("name", list(W.ORDER) + list(EXTRA))
def test_auto_is_the_fastest_built_projection(name):
    wl = W.WORKLOADS[name] if name in W.WORKLOADS else EXTRA[name]
    x, taps = W.make(wl)
    nrot = max(2, min(6, -(-2 * (256 << 20) // wl.algorithmic_bytes)))
    dxs = [torch.from_numpy(x).cuda() for _ in range(nrot)]
    dys = [torch.empty(wl.y_shape, dtype=torch.float32, device="cuda") for _ in range(nrot)]
    if wl.ndim == 1:
        projs = [p for p in ("FBS", "SBM", "BFS", "BSM", "FSM", "FFS") if B.sys_conv1d_has(p, wl.k_shape[0])]
        conv = B.sys_conv1d
    else:
        projs = [p for p in ("FBS", "SBM", "BFS") if B.sys_conv2d_has(p, *wl.k_shape)]
        conv = B.sys_conv2d
    launches = 200 if wl.algorithmic_bytes < (16 << 20) else 30 if wl.n_taps < 5_000_000_000 else 8

    small = wl.algorithmic_bytes < (16 << 20)
    graphs = {}

    def runner(proj):
        if not small:
            return lambda i: conv(dxs[i % nrot], taps, dys[i % nrot], projection=proj)
        conv(dxs[0], taps, dys[0], projection=proj)                  # load the code object outside the capture
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(100):
                conv(dxs[i % nrot], taps, dys[i % nrot], projection=proj)
        graphs[proj] = g
        return lambda i: g.replay()

    if small:
        launches = 5                                                 # replays of 100 launches each
    best = {p: float("inf") for p in projs + ["AUTO"]}
    runners = {p: runner(p) for p in best}
    for p in best:                                                   # warm-up: code objects, clocks
        _batch_time(runners[p], 10 if not small else 2)
    for _ in range(5):
        for p in best:
            best[p] = min(best[p], _batch_time(runners[p], launches) / (100 if small else 1))
    fastest = min(projs, key=lambda p: best[p])
    report = ", ".join(f"{p} {best[p]:.2f}" for p in best)
    print(f"{name}: {report} us", flush=True)
    assert best["AUTO"] <= TOLERANCE * best[fastest], f"{name}: AUTO {best['AUTO']:.2f} us, {fastest} {best[fastest]:.2f} us ({report})"
