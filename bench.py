#!/usr/bin/env python3
"""Benchmark of libsysconv on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extras] [--no-cpu]
    python bench.py --design-space      # the six 1-D designs of Table 2 at n = 2^26, k = 2, 5, 16
    python bench.py --paper-shape       # the grid of the paper's Section 6 experiment (671 M outputs per case)

A step is one pass of the hot path -- weight residency, input load, systolic time
loop, output store -- over the large 1-D workload (n = 2^26 fp32 inputs, 16
taps), launched through the C ABI with inputs already resident in HBM.  The
single JSON line printed at the end carries

  value        algorithmic GB/s of that step (4 B per input + 4 B per output + taps,
               divided by wall time between two device synchronisations)
  roofline     the same bytes over the kernel's average duration on the GPU's clock (HIP
               events on the launch stream at the start and the end of the timed
               region and at four points in between; elapsed time / launches),
               against the 8 TB/s HBM peak; `traffic` is the HBM byte
               count of one launch from hardware counters when a calibrated
               reading is stored in profiles/, else null
  roofline_alu the same for the 8192^2, 11x11 workload, which is bound by the vector ALUs:
               2 x multiply-adds / kernel time against the 78.6 TFLOP/s fp32 vector peak
  roofline_mfma that workload through the opt-in matrix-core projection: issued MFMA flops against
               the 2.5 PFLOP/s dense fp16 peak, with the fraction of them the definition needs
  roofline_2d  the 4096^2, 5x5 workload (bound by HBM): its fastest projection against the 8 TB/s peak, with the
               output rows packed tightly and on 128-byte lines
  cpu_baseline the CPU oracle (plain C, fp64) timed here on the host cores
  also         all five workloads and every projection built for them, each with
               GB/s, Gtap/s and its fraction of the HBM and fp32-FMA peaks, a plain
               dwordx4 copy of the same footprint, and for the launch-bound ones the
               time per launch when 100 launches are replayed from a HIP graph; for the
               two large 2-D workloads also the fastest projection with the output rows
               on 128-byte lines (y_pitch_floats: a pitch the caller is free to choose)

Paper context (not a target, not comparable): on an Intel GEN9.5 iGPU the paper's
best software-systolic designs ran up to 59 % faster than that GPU's hardware
samplers; it reports no absolute throughput.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
FMA_PEAK_G = 39321.6             # 256 CUs x 64 lanes x 2.4 GHz, one v_fmac_f32 per lane-clock (= 78.6 TFLOP/s)
HEADLINE = "conv1d_64m_k16"
MALL_BYTES = 256 << 20           # last-level cache in front of HBM: rotate buffers past it


def _parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--projection", default="AUTO")
    ap.add_argument("--no-extras", action="store_true", help="skip the other workloads / projections")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--design-space", action="store_true",
                    help="only time the six 1-D designs of the paper's Table 2 at n=2^26 for k in {2, 5, 16} "
                         "(the paper's Table 3 uses k = 2 and 5) and print that table as JSON")
    ap.add_argument("--paper-shape", action="store_true",
                    help="only time the grid of the paper's Section 6 experiment: 10 Mi 'threads' of 16x4 outputs each "
                         "(671 M outputs), 1-D k in {2, 5} at stride 1 (six designs) and stride 2 (FBS), 2-D 2x2 and "
                         "5x5 at stride 1 (SBM, FBS, BFS) and stride 2 (FBS); throughput = outputs / time, as in the "
                         "paper; prints JSON")
    ap.add_argument("--size-sweep", action="store_true",
                    help="only time the 5x5 convolution (every projection built for it) and a plain copy of the same "
                         "footprint on square images from 2048^2 to 16384^2, and fit time = t0 + bytes / rate to each: "
                         "how much of the 4096^2 workload's time is start-up and tail, and what rate the kernels "
                         "approach on large images; prints JSON")
    return ap.parse_args()


def kernel_source_hash() -> str:
    """Fingerprint of the kernel sources (csrc/*.hip, *.h): counter readings stored under profiles/
    carry the fingerprint of the sources they were taken with."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2010_15884_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def _stored_traffic(kernel_key: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by
    the copy kernel's reading); kept as `traffic_bytes <key> <bytes>` lines in profiles/hbm_traffic.txt
    together with the fingerprint of the kernel sources they were measured on.  Returns
    (bytes or None, provenance): a reading taken on other sources than the ones now in the tree
    is not reported as this run's traffic."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    prov = {"file": "profiles/hbm_traffic.txt", "measured_on_sources": None, "sources_now": kernel_source_hash()}
    if not os.path.exists(path):
        return None, prov
    value = None
    for line in open(path):
        m = re.match(r"traffic_bytes\s+(\S+)\s+(\d+)", line.strip())
        if m and m.group(1) == kernel_key:
            value = int(m.group(2))
        m = re.match(r"source_hash\s+(\S+)", line.strip())
        if m:
            prov["measured_on_sources"] = m.group(1)
    prov["stale"] = prov["measured_on_sources"] != prov["sources_now"]
    if prov["stale"]:
        prov["stale_reading"] = value
        value = None
    return value, prov


def main() -> int:
    args = _parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2010_15884_amd import binding as B
    from paper_2010_15884_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.lib()                                       # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    def rotation(wl):
        per_pass = wl.algorithmic_bytes
        return max(2, min(6, -(-2 * MALL_BYTES // per_pass)))

    def make_launcher(wl, proj, x_host, taps, y_pitch=None):
        nrot = rotation(wl)
        dxs = [torch.from_numpy(x_host).cuda() for _ in range(nrot)]
        if y_pitch is None:
            dys = [torch.empty(wl.y_shape, dtype=torch.float32, device="cuda") for _ in range(nrot)]
        else:                                               # rows y_pitch floats apart; the result is the left part
            dys = [torch.empty((wl.y_shape[0], y_pitch), dtype=torch.float32, device="cuda")[:, :wl.y_shape[1]]
                   for _ in range(nrot)]
        state = {"i": 0}
        conv = B.sys_conv1d if wl.ndim == 1 else B.sys_conv2d

        def launch():
            i = state["i"] = (state["i"] + 1) % nrot
            conv(dxs[i], taps, dys[i], projection=proj)
        return launch, (dxs, dys)

    def time_launches(launch, steps, warmup):
        """Time `steps` back-to-back launches.  Returns (wall seconds between two device synchronisations,
        mean seconds per launch on the GPU's clock, median of the per-batch means).

        HIP events are recorded on the launch stream before the first launch, after the last one and at up to
        four points in between -- not around every launch: an event pair per launch costs 7 us per step here
        (n = 2^26, k = 16: 93.6 us per step with pairs, 86.2 us without, 86.5 us in the rocprofv3 kernel
        trace), which would be charged to the kernel.  A launch's duration is therefore the length of its
        batch divided by the launches in it; the few gaps between back-to-back kernels are included."""
        # the GPU drops its clocks while the host prepares inputs: keep it busy for ~50 ms
        # first so that the timed launches see steady-state clocks, then the W warm-up steps
        t_spin = time.perf_counter()
        while time.perf_counter() - t_spin < 0.05:
            for _ in range(8):
                launch()
            torch.cuda.synchronize()
        for _ in range(warmup):
            launch()
        n_batches = min(5, steps)
        bounds = [steps * i // n_batches for i in range(n_batches + 1)]
        evs = [torch.cuda.Event(enable_timing=True) for _ in bounds]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        evs[0].record(stream)
        for bi in range(n_batches):
            for _ in range(bounds[bi], bounds[bi + 1]):
                launch()
            evs[bi + 1].record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        total = evs[0].elapsed_time(evs[-1]) * 1e-3
        per_batch = sorted(evs[bi].elapsed_time(evs[bi + 1]) * 1e-3 / (bounds[bi + 1] - bounds[bi])
                           for bi in range(n_batches))
        return wall, total / steps, per_batch[len(per_batch) // 2]

    if args.size_sweep:
        sides = (2048, 2896, 4096, 5792, 8192, 11584, 16384)
        base = W.WORKLOADS["conv2d_4k_5x5"]
        series = {}
        rows = []
        for side in sides:
            wk = W.Workload(f"conv2d_{side}_5x5", 2, (side, side), base.k_shape, base.x_range, base.w_range, base.seed)
            nrot = rotation(wk)
            g = torch.Generator(device="cuda")
            g.manual_seed(base.seed)
            dxs = [torch.empty(wk.x_shape, dtype=torch.float32, device="cuda").uniform_(0.0, 1.0, generator=g)
                   for _ in range(nrot)]
            dys = [torch.empty(wk.y_shape, dtype=torch.float32, device="cuda") for _ in range(nrot)]
            _, taps = W.make(base, x_shape=(8, 8))
            st = {"i": 0}
            n_copy = wk.algorithmic_bytes // 8
            flat_src = [d.view(-1)[:n_copy] for d in dxs]
            flat_dst = [torch.empty(n_copy, dtype=torch.float32, device="cuda") for _ in range(nrot)]

            def copy_launch():
                i = st["i"] = (st["i"] + 1) % nrot
                B.sys_copy_f32(flat_src[i], flat_dst[i])
            steps = 40 if side <= 8192 else 12
            _, c_mean, _ = time_launches(copy_launch, steps, 3)
            row = {"side": side, "algorithmic_bytes": wk.algorithmic_bytes, "copy_us": round(c_mean * 1e6, 2)}
            series.setdefault("copy", []).append((wk.algorithmic_bytes, c_mean))
            del flat_dst
            for proj in ("BFS", "SBM", "FBS", "MFMA"):
                def launch():
                    i = st["i"] = (st["i"] + 1) % nrot
                    B.sys_conv2d(dxs[i], taps, dys[i], projection=proj)
                _, k_mean, _ = time_launches(launch, steps, 3)
                row[f"{proj}_us"] = round(k_mean * 1e6, 2)
                row[f"{proj}_frac_hbm_peak"] = round(wk.algorithmic_bytes / k_mean / 1e9 / HBM_PEAK_GBS, 4)
                series.setdefault(proj, []).append((wk.algorithmic_bytes, k_mean))
            rows.append(row)
            print(json.dumps(row), file=sys.stderr, flush=True)
            del dxs, dys, flat_src
            torch.cuda.empty_cache()
        fits = {}
        for name, pts in series.items():
            b = np.array([p[0] for p in pts], dtype=np.float64)
            t = np.array([p[1] for p in pts], dtype=np.float64)
            slope, t0 = np.polyfit(b, t, 1)                      # t = t0 + bytes * slope
            fits[name] = {"t0_us": round(t0 * 1e6, 2), "rate_GB/s": round(1e-9 / slope, 1),
                          "rate_frac_hbm_peak": round(1e-9 / slope / HBM_PEAK_GBS, 4),
                          "max_residual_us": round(float(np.max(np.abs(t - (t0 + slope * b)))) * 1e6, 2)}
        print(json.dumps({"size_sweep_5x5": rows, "fit": fits, "data": "synthetic (uniform fp32 drawn on the device)",
                          "note": "least-squares fit of kernel time = t0 + algorithmic bytes / rate over the seven sizes"}))
        return 0

    if args.design_space:
        from paper_2010_15884_amd import schedule_model as sm
        paper_rel = {"SBM": (157, 147), "BSM": (67, 49), "FSM": (56, 39), "BFS": (56, 48), "FFS": (33, 30),
                     "FBS": (159, 157)}                    # Table 3: % of the hardware sampler at k = 2, 5
        wl = W.WORKLOADS[HEADLINE]
        x_host, _ = W.make(wl)
        rows = []
        for k in (2, 5, 16):
            taps = W.uniform_f32(np.random.default_rng(15884 + k), -1.0, 1.0, (k,))
            wk = W.Workload(f"conv1d_64m_k{k}", 1, wl.x_shape, (k,), wl.x_range, wl.w_range, wl.seed)
            t_fbs = None
            for proj in ("FBS", "SBM", "BFS", "BSM", "FSM", "FFS"):
                ln, kp = make_launcher(wk, proj, x_host, taps)
                _, k_mean, _ = time_launches(ln, 10, 2)
                del ln, kp
                t_fbs = k_mean if proj == "FBS" else t_fbs
                row = {"k": k, "design": proj, "kernel_us": round(k_mean * 1e6, 1),
                       "GB/s": round(wk.algorithmic_bytes / k_mean / 1e9, 1),
                       "Gtap/s": round(wk.n_taps / k_mean / 1e9, 1),
                       "relative_to_FBS": round(t_fbs / k_mean, 3),
                       "model_utilisation_wave64": round(sm.wave64(proj, k)["utilisation"], 3)}
                if k in (2, 5):
                    p = paper_rel[proj][0 if k == 2 else 1]
                    row["paper_relative_to_FBS"] = round(p / paper_rel["FBS"][0 if k == 2 else 1], 3)
                rows.append(row)
            # the same six designs through the generic space-time-transform kernel (one PE per lane,
            # nothing specialised): what the general code shape of Section 4.1 costs on this machine
            for proj in ("FBS", "SBM", "BFS", "BSM", "FSM", "FFS"):
                design = B.named_design(proj)
                dxs = [torch.from_numpy(x_host).cuda() for _ in range(2)]
                dys = [torch.empty(wk.y_shape, dtype=torch.float32, device="cuda") for _ in range(2)]
                state = {"i": 0}

                def launch():
                    i = state["i"] = (state["i"] + 1) % 2
                    B.sys_conv1d_stt(dxs[i], taps, design, dys[i])
                _, k_mean, _ = time_launches(launch, 5, 1)
                del dxs, dys
                rows.append({"k": k, "design": f"generic({proj})", "kernel_us": round(k_mean * 1e6, 1),
                             "GB/s": round(wk.algorithmic_bytes / k_mean / 1e9, 1),
                             "Gtap/s": round(wk.n_taps / k_mean / 1e9, 1),
                             "relative_to_FBS": round(t_fbs / k_mean, 3)})
        print(json.dumps({"design_space_1d": rows, "n": wl.x_shape[0], "data": "synthetic",
                          "note": "paper column: Table 3 (Intel GEN9.5, relative to its hardware sampler), "
                                  "rescaled to FBS = 1; context, not a target"}))
        return 0

    if args.paper_shape:
        threads, per_thread = 10 * (1 << 20), 16 * 4        # Section 6: more than ten million threads, 16*4 outputs each
        outputs = threads * per_thread
        paper_1d = {"SBM": (157, 147), "BSM": (67, 49), "FSM": (56, 39), "BFS": (56, 48), "FFS": (33, 30),
                    "FBS": (159, 157)}                      # Table 3, % of the hardware sampler (k = 2, 5)
        paper_2d = {"SBM": (92, 20), "FBS": (114, 24)}      # Table 5 (2x2, 5x5)
        rows = []

        def device_uniform(shape, lo, hi, seed):
            # inputs of 2.5 - 10 GiB: drawn on the device (seeded), not shipped from the host
            g = torch.Generator(device="cuda")
            g.manual_seed(seed)
            return torch.empty(shape, dtype=torch.float32, device="cuda").uniform_(lo, hi, generator=g)

        def timed(launch, read_floats, taps_per_out, row):
            _, k_mean, _ = time_launches(launch, 5, 1)
            row.update({"kernel_us": round(k_mean * 1e6, 1), "Goutputs/s": round(outputs / k_mean / 1e9, 2),
                        "GB/s": round(4 * (read_floats + outputs) / k_mean / 1e9, 1),
                        "Gtap/s": round(outputs * taps_per_out / k_mean / 1e9, 1)})
            rows.append(row)
            print(json.dumps(row), file=sys.stderr, flush=True)

        # two buffer pairs in rotation: >= 5 GB per pass, far past the memory-side cache
        for stride in (1, 2):
            for ki, k in enumerate((2, 5)):
                taps = W.uniform_f32(np.random.default_rng(15884 + k), -1.0, 1.0, (k,))
                n = stride * (outputs - 1) + k
                dxs = [device_uniform((n,), -1.0, 1.0, 158846 + i) for i in range(2)]
                dys = [torch.empty((outputs,), dtype=torch.float32, device="cuda") for _ in range(2)]
                st = {"i": 0}
                for proj in (("FBS", "SBM", "BFS", "BSM", "FSM", "FFS") if stride == 1 else ("FBS",)):
                    def launch():
                        i = st["i"] = (st["i"] + 1) % 2
                        B.sys_conv1d_strided(dxs[i], taps, stride, dys[i], projection=proj)
                    row = {"conv": "1-D", "k": k, "stride": stride, "design": proj}
                    if stride == 1:
                        row["paper_relative_to_FBS"] = round(paper_1d[proj][ki] / paper_1d["FBS"][ki], 3)
                    timed(launch, n, k, row)
                del dxs, dys
        oh, ow = 16384, outputs // 16384
        for stride in (1, 2):
            for ki, kk in enumerate((2, 5)):
                f = W.uniform_f32(np.random.default_rng(15884 + 10 * kk), -1.0, 1.0, (kk, kk))
                h, w_img = stride * (oh - 1) + kk, stride * (ow - 1) + kk
                dxs = [device_uniform((h, w_img), 0.0, 1.0, 158856 + i) for i in range(2)]
                dys = [torch.empty((oh, ow), dtype=torch.float32, device="cuda") for _ in range(2)]
                st = {"i": 0}
                for proj in (("FBS", "SBM", "BFS") if stride == 1 else ("FBS",)):
                    def launch():
                        i = st["i"] = (st["i"] + 1) % 2
                        B.sys_conv2d_strided(dxs[i], f, stride, dys[i], projection=proj)
                    row = {"conv": "2-D", "k": f"{kk}x{kk}", "stride": stride, "design": proj}
                    if stride == 1 and proj in paper_2d:
                        row["paper_relative_to_FBS"] = round(paper_2d[proj][ki] / paper_2d["FBS"][ki], 3)
                    timed(launch, h * w_img, kk * kk, row)
                del dxs, dys
                torch.cuda.empty_cache()
        ref = {(r["conv"], r["k"], r["stride"]): r["kernel_us"] for r in rows if r["design"] == "FBS"}
        for r in rows:
            r["relative_to_FBS"] = round(ref[(r["conv"], r["k"], r["stride"])] / r["kernel_us"], 3)
        print(json.dumps({"paper_shape": rows, "threads": threads, "outputs_per_thread": per_thread,
                          "outputs": outputs, "data": "synthetic",
                          "note": "paper columns: Tables 3 and 5 (Intel GEN9.5, relative to its hardware sampler), "
                                  "rescaled to FBS = 1; context, not a target; the paper prints no stride-2 figures"}))
        return 0

    # ------------------------------------------------------------ headline step
    wl = W.WORKLOADS[HEADLINE]
    x_host, taps = W.make(wl)
    launch, keep = make_launcher(wl, args.projection, x_host, taps)
    wall, kern_mean, kern_med = time_launches(launch, args.steps, args.warmup)
    ms_per_step = 1e3 * wall / args.steps
    value = wl.algorithmic_bytes / (wall / args.steps) / 1e9
    achieved = wl.algorithmic_bytes / kern_mean / 1e9
    del keep, launch
    torch.cuda.empty_cache()

    # a plain dwordx4 copy with the same footprint (2^26 floats read, 2^26 written): what the
    # memory system gives a streaming kernel, and the known-traffic kernel for counter calibration
    n_copy = wl.x_shape[0]
    srcs = [torch.empty(n_copy, dtype=torch.float32, device="cuda").normal_() for _ in range(2)]
    dsts = [torch.empty(n_copy, dtype=torch.float32, device="cuda") for _ in range(2)]
    cstate = {"i": 0}

    def copy_launch():
        i = cstate["i"] = (cstate["i"] + 1) % 2
        B.sys_copy_f32(srcs[i], dsts[i])
    _, copy_mean, _ = time_launches(copy_launch, args.steps, args.warmup)
    copy_gbs = 8 * n_copy / copy_mean / 1e9
    del srcs, dsts
    torch.cuda.empty_cache()

    # the kernel behind the headline projection (AUTO picks FBS at 16 taps)
    head_proj = "FBS" if args.projection.upper() == "AUTO" else args.projection.upper()
    head_traffic, head_prov = _stored_traffic(f"conv1d_{head_proj.lower()}_k16_n64m")
    head_kernel = {"FBS": "conv1d_fbs_kernel<16>", "SBM": "conv1d_sbm_kernel<16>", "BFS": "conv1d_bfs_kernel<16>",
                   "BSM": "conv1d_array_kernel<0>", "FSM": "conv1d_array_kernel<1>",
                   "FFS": "conv1d_array_kernel<2>"}[head_proj]
    result = {
        "metric": "conv GB/s (algorithmic bytes / time), 1-D valid convolution n=2^26 K=16 fp32",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic (seeded uniform fp32, see paper_2010_15884_amd/workloads.py)",
        "config": {"workload": HEADLINE, "n": wl.x_shape[0], "taps": wl.k_shape[0],
                   "projection": args.projection, "algorithmic_bytes": wl.algorithmic_bytes,
                   "gtap_per_s": round(wl.n_taps / (wall / args.steps) / 1e9, 1)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": head_traffic, "traffic_source": head_prov,
                     "kernel": head_kernel, "kernel_us_mean": round(kern_mean * 1e6, 2),
                     "kernel_us_median": round(kern_med * 1e6, 2),
                     "copy_same_footprint_GB/s": round(copy_gbs, 1),
                     "frac_of_copy": round(achieved / copy_gbs, 3)},
        "paper_context": "Intel GEN9.5, fp32: best software-systolic designs up to 59% faster than that GPU's "
                         "hardware samplers (relative figure only; not a target)",
    }

    # ----------------------------------------------------- the other workloads
    if not args.no_extras:
        also = []
        for name in W.ORDER:
            w2 = W.WORKLOADS[name]
            xh, tp = W.make(w2)
            steps = 30 if w2.n_taps < 5_000_000_000 else 10
            # plain copy of the same footprint (half read, half written)
            n_copy = max(1, w2.algorithmic_bytes // 8)
            nrot = rotation(w2)
            srcs = [torch.empty(n_copy, dtype=torch.float32, device="cuda").normal_() for _ in range(nrot)]
            dsts = [torch.empty(n_copy, dtype=torch.float32, device="cuda") for _ in range(nrot)]
            st = {"i": 0}

            def copy_launch():
                i = st["i"] = (st["i"] + 1) % nrot
                B.sys_copy_f32(srcs[i], dsts[i])
            _, c_mean, _ = time_launches(copy_launch, steps, 3)
            copy_gbs = 8 * n_copy / c_mean / 1e9
            del srcs, dsts
            for proj in ("FBS", "SBM", "BFS", "BSM", "FSM", "FFS", "MFMA"):
                has = B.sys_conv1d_has(proj, w2.k_shape[0]) if w2.ndim == 1 else B.sys_conv2d_has(proj, *w2.k_shape)
                if not has:
                    continue
                ln, kp = make_launcher(w2, proj, xh, tp)
                _, k_mean, k_med = time_launches(ln, steps, 3)
                gbs = w2.algorithmic_bytes / k_mean / 1e9
                gtap = w2.n_taps / k_mean / 1e9
                row = {"workload": name, "projection": proj, "kernel_us_mean": round(k_mean * 1e6, 2),
                       "kernel_us_median": round(k_med * 1e6, 2), "GB/s": round(gbs, 1),
                       "Gtap/s": round(gtap, 1), "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                       "frac_fma_peak": round(gtap / FMA_PEAK_G, 4),
                       "copy_GB/s_same_footprint": round(copy_gbs, 1),
                       "frac_of_copy": round(gbs / copy_gbs, 3)}
                if k_mean < 20e-6:
                    # launch-bound: the same launches recorded into a HIP graph, 100 per replay
                    graph = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(graph):
                        for _ in range(100):
                            ln()
                    _, g_mean, _ = time_launches(graph.replay, 10, 2)
                    row["graph_us_per_launch"] = round(g_mean * 1e6 / 100, 2)
                    del graph
                also.append(row)
                del ln, kp
            # "Valid" outputs are kw-1 columns narrower than the image, so with rows packed tightly most of them start
            # inside a 128-byte line and every wavefront's 1 KB store straddles lines.  The boundary lets the caller
            # choose the pitch: the fastest projection again with the output rows on 128-byte lines (same algorithmic
            # bytes: the padding is never written).
            if w2.ndim == 2 and w2.y_shape[1] % 32 and w2.algorithmic_bytes > (16 << 20):
                mine = [r for r in also if r["workload"] == name and r["projection"] != "MFMA"]
                best = min(mine, key=lambda r: r["kernel_us_mean"])
                pitch = -(-w2.y_shape[1] // 32) * 32
                ln, kp = make_launcher(w2, best["projection"], xh, tp, y_pitch=pitch)
                _, k_mean, k_med = time_launches(ln, steps, 3)
                gbs = w2.algorithmic_bytes / k_mean / 1e9
                also.append({"workload": name, "projection": best["projection"], "y_pitch_floats": pitch,
                             "kernel_us_mean": round(k_mean * 1e6, 2), "kernel_us_median": round(k_med * 1e6, 2),
                             "GB/s": round(gbs, 1), "Gtap/s": round(w2.n_taps / k_mean / 1e9, 1),
                             "frac_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                             "frac_fma_peak": round(w2.n_taps / k_mean / 1e9 / FMA_PEAK_G, 4),
                             "copy_GB/s_same_footprint": round(copy_gbs, 1), "frac_of_copy": round(gbs / copy_gbs, 3),
                             "note": "same workload, output rows 128-byte aligned (caller-chosen pitch)"})
                del ln, kp
        result["also"] = also
        # the one workload that is bound by the vector ALUs, not by HBM: its own roofline object
        # (121 multiply-adds per 8 bytes; peak = 256 CUs x 64 lanes x 2.4 GHz x 2 flop = 78.6 TFLOP/s fp32)
        alu = [r for r in also if r["workload"] == "conv2d_8k_11x11" and r["projection"] != "MFMA" and "y_pitch_floats" not in r]
        if alu:
            best = max(alu, key=lambda r: r["Gtap/s"])
            kern = {"SBM": "conv2d_sbm_kernel<11, 11, 1>", "BFS": "conv2d_bfs_kernel<11, 11, 1>",
                    "FBS": "conv2d_fbs_kernel<2>"}[best["projection"]]
            alu_traffic, alu_prov = _stored_traffic(f"conv2d_{best['projection'].lower()}_11x11_8k")
            # what the vector ALUs sustain with nothing in the way: the register-only yard-stick, 8 wavefronts per SIMD
            ybuf = torch.empty(2048 * 256, dtype=torch.float32, device="cuda")
            fmas = {"n": 0}

            def alu_launch():
                fmas["n"] = B.sys_alu_yardstick_f32(ybuf, 2048, 500)
            _, y_mean, _ = time_launches(alu_launch, 10, 2)
            yard_g = fmas["n"] / y_mean / 1e9
            result["roofline_alu"] = {
                "workload": "conv2d_8k_11x11", "projection": best["projection"], "kernel": kern, "bound": "alu",
                "achieved": round(2 * best["Gtap/s"] / 1e3, 2), "peak": round(2 * FMA_PEAK_G / 1e3, 1),
                "unit": "TFLOP/s", "frac": round(best["Gtap/s"] / FMA_PEAK_G, 4),
                "frac_of_published_fp32_vector_peak_157.3": round(2 * best["Gtap/s"] / 1e3 / 157.3, 4),
                "measured_fmac_yardstick_TFLOP/s": round(2 * yard_g / 1e3, 2),
                "frac_of_measured_yardstick": round(best["Gtap/s"] / yard_g, 4),
                "traffic": alu_traffic, "traffic_source": alu_prov,
                "kernel_us_mean": best["kernel_us_mean"],
                "note": "peak = 256 CUs x 64 lanes x 2.4 GHz x 2 flop (one v_fmac_f32 per lane-clock); the published "
                        "157.3 TFLOP/s counts packed fp32 instructions, which this build does not use"}
        # the same workload on the matrix cores (opt-in projection): issued MFMA flops against the dense fp16 peak,
        # and how many of them are the definition's own multiply-adds
        mf = [r for r in also if r["workload"] == "conv2d_8k_11x11" and r["projection"] == "MFMA"]
        if mf:
            r = mf[0]
            w5 = W.WORKLOADS["conv2d_8k_11x11"]
            ns = (w5.k_shape[0] + 4) // 2                    # instructions per product and 4 x 64 block of outputs
            issued_macs_per_output = 3 * ns * 16 * 16 * 32 / 256.0
            t = r["kernel_us_mean"] * 1e-6
            achieved = 2 * issued_macs_per_output * w5.n_outputs / t / 1e12
            mf_traffic, mf_prov = _stored_traffic("conv2d_mfma_11x11_8k")
            result["roofline_mfma"] = {
                "workload": "conv2d_8k_11x11", "projection": "MFMA", "kernel": f"conv2d_mfma_kernel<{ns}, 3>",
                "bound": "mfma", "achieved": round(achieved, 1), "peak": 2500.0, "unit": "TFLOP/s",
                "frac": round(achieved / 2500.0, 4),
                "useful_fraction": round(w5.k_shape[0] * w5.k_shape[1] / issued_macs_per_output, 4),
                "useful_TFLOP/s": round(2 * r["Gtap/s"] / 1e3, 2),
                "frac_hbm_peak": r["frac_hbm_peak"], "traffic": mf_traffic, "traffic_source": mf_prov,
                "kernel_us_mean": r["kernel_us_mean"],
                "note": "v_mfma_f32_16x16x32_f16 on split fp16 operands (3 products); useful_fraction = kh*kw "
                        "multiply-adds of the definition / multiply-adds issued (Toeplitz zeros and the split)"}

        # the large 2-D workload that is bound by HBM: its own roofline object (best projection, tight and aligned pitch)
        c4 = [r for r in also if r["workload"] == "conv2d_4k_5x5" and r["projection"] != "MFMA"]
        if c4:
            tight = min((r for r in c4 if "y_pitch_floats" not in r), key=lambda r: r["kernel_us_mean"])
            kern = {"BFS": "conv2d_bfs_block_kernel<5, 5, 2>", "SBM": "conv2d_sbm_block_kernel<5, 5, 4>",
                    "FBS": "conv2d_fbs_static_kernel<5, 5, 2>"}[tight["projection"]]
            t_traffic, t_prov = _stored_traffic(f"conv2d_{tight['projection'].lower()}_5x5_4k")
            obj = {"workload": "conv2d_4k_5x5", "projection": tight["projection"], "kernel": kern, "bound": "hbm",
                   "achieved": tight["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": tight["frac_hbm_peak"],
                   "traffic": t_traffic, "traffic_source": t_prov, "kernel_us_mean": tight["kernel_us_mean"],
                   "frac_of_copy": tight["frac_of_copy"]}
            al = [r for r in c4 if "y_pitch_floats" in r]
            if al:
                obj["aligned_output_pitch"] = {"y_pitch_floats": al[0]["y_pitch_floats"], "projection": al[0]["projection"],
                                               "achieved": al[0]["GB/s"], "frac": al[0]["frac_hbm_peak"],
                                               "frac_of_copy": al[0]["frac_of_copy"],
                                               "kernel_us_mean": al[0]["kernel_us_mean"]}
            result["roofline_2d"] = obj

    # ---------------------------------------------------------- CPU baseline
    if not args.no_cpu:
        import oracle
        threads = oracle.threads_used(min(16, os.cpu_count() or 1))

        def passes(nthreads, budget_s):
            """Whole passes of the headline workload through the oracle for about budget_s seconds."""
            oracle.conv1d(x_host, taps, nthreads)                       # first touch of the library and the pages
            reps, t0 = 0, time.perf_counter()
            while True:
                oracle.conv1d(x_host, taps, nthreads)
                reps += 1
                el = time.perf_counter() - t0
                if el >= budget_s or reps >= 200:
                    return reps, el

        reps, cpu_s = passes(threads, 2.0)                              # ~30 core-seconds of CPU work
        reps1, cpu1_s = passes(1, 2.0)
        result["cpu_baseline"] = {
            "value": round(reps * wl.algorithmic_bytes / cpu_s / 1e9, 3), "unit": "GB/s", "cores": threads,
            "kind": "oracle",
            "sample": f"{reps} passes of the whole {HEADLINE} workload ({wl.n_taps / 1e9:.2f} G fp64 multiply-adds "
                      f"each), oracle/conv_oracle.c with {threads} OpenMP threads, result array allocated per pass",
            "seconds": round(cpu_s, 3),
            "single_thread": {"value": round(reps1 * wl.algorithmic_bytes / cpu1_s / 1e9, 3), "unit": "GB/s",
                              "cores": 1, "sample": f"{reps1} passes of the same workload on one thread",
                              "seconds": round(cpu1_s, 3)},
        }

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
