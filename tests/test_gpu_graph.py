"""The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation, no memset),
so a caller may record them into a HIP graph.  Replays must give what eager calls give, every time."""
import numpy as np
import pytest
import torch

from gpu_common import TOL, dev, err1d, err2d
from paper_2010_15884_amd import binding as B
from paper_2010_15884_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_captured_launches_replay_like_eager_calls():
    n, k = 65536, 5
    h, wd, kk = 300, 700, 5
    x, w = W.random_case(1, (n,), (k,))
    img, f = W.random_case(2, (h, wd), (kk, kk), x_range=(0.0, 1.0))
    dx, dimg = dev(x), dev(img)
    y1 = torch.zeros(n - k + 1, dtype=torch.float32, device="cuda")
    y1s = torch.zeros((n - k) // 2 + 1, dtype=torch.float32, device="cuda")
    ygen = torch.zeros(n - k + 1, dtype=torch.float32, device="cuda")
    y2 = {p: torch.zeros((h - kk + 1, wd - kk + 1), dtype=torch.float32, device="cuda") for p in ("FBS", "BFS", "SBM")}
    design = B.named_design("FSM")

    def enqueue():
        for p in ("FBS", "SBM", "BFS", "BSM"):
            B.sys_conv1d(dx, w, y1, projection=p)                  # the last one's result stays in y1
        B.sys_conv1d_strided(dx, w, 2, y1s, projection="FBS")
        B.sys_conv1d_stt(dx, w, design, ygen)
        for p, out in y2.items():
            B.sys_conv2d(dimg, f, out, projection=p)

    enqueue()                                                       # warm up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        enqueue()
    for rep in range(4):
        # new contents in the same buffers, eager work and a synchronisation between the replays
        x, _ = W.random_case(10 + rep, (n,), (k,))
        img, _ = W.random_case(20 + rep, (h, wd), (kk, kk), x_range=(0.0, 1.0))
        dx.copy_(dev(x))
        dimg.copy_(dev(img))
        for t in (y1, y1s, ygen, *y2.values()):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert err1d(y1.cpu().numpy(), x, w) <= TOL, rep
        assert err1d(ygen.cpu().numpy(), x, w) <= TOL, rep
        assert np.array_equal(y1s.cpu().numpy(), B.sys_conv1d_strided(dx, w, 2, projection="FBS").cpu().numpy()), rep
        for p, out in y2.items():
            assert err2d(out.cpu().numpy(), img, f) <= TOL, (rep, p)
            assert np.array_equal(out.cpu().numpy(), B.sys_conv2d(dimg, f, projection=p).cpu().numpy()), (rep, p)


def test_taps_are_frozen_at_capture_time():
    # the taps travel in the kernel-argument block, so a replay uses the taps of the captured call
    n, k = 20000, 7
    x, w = W.random_case(3, (n,), (k,))
    dx = dev(x)
    y = torch.zeros(n - k + 1, dtype=torch.float32, device="cuda")
    w_live = w.copy()
    B.sys_conv1d(dx, w_live, y, projection="FBS")
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.sys_conv1d(dx, w_live, y, projection="FBS")
    w_live[:] = 0.0                                                 # the caller's array changes after the capture
    y.fill_(float("nan"))
    torch.cuda.synchronize()
    g.replay()
    torch.cuda.synchronize()
    assert err1d(y.cpu().numpy(), x, w) <= TOL
