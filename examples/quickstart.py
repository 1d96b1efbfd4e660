#!/usr/bin/env python3
"""The Python binding in a dozen lines (needs an MI355X and a built libsysconv.so).

    python -m paper_2010_15884_amd.build && python examples/quickstart.py
"""
import os
import sys

import numpy as np
import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_2010_15884_amd import binding as sysconv  # noqa: E402

x = torch.rand(1 << 20, device="cuda") * 2 - 1            # signal in device memory
w = np.array([0.25, 0.5, 0.25], np.float32)               # taps stay on the host

y = sysconv.sys_conv1d(x, w)                              # AUTO picks the projection
y_sbm = sysconv.sys_conv1d(x, w, projection="SBM")        # or name one of the paper's designs
y_s2 = sysconv.sys_conv1d_strided(x, w, 2)                # y[c] = sum_q x[2c+q] w[q]
print("1-D:", tuple(y.shape), "max |FBS - SBM| =", float((y - y_sbm).abs().max()),
      " stride 2:", tuple(y_s2.shape))

# a design the paper does not list, written down as data: SBM whose sums move every second step
half_speed = sysconv.stt_design(alloc=(1, 1), sched=(1, 2), dep_x=(-1, 1), dep_w=None, dep_z=(0, 1))
print("design check:", sysconv.status_string(sysconv.sys_stt_check(half_speed, len(w))))
y_gen = sysconv.sys_conv1d_stt(x, w, half_speed)
print("generic kernel: max |generic - FBS| =", float((y_gen - y).abs().max()))

img = torch.rand((2048, 2048), device="cuda")
f = np.outer([1, 4, 6, 4, 1], [1, 4, 6, 4, 1]).astype(np.float32) / 256
out = sysconv.sys_conv2d(img, f)                          # 5x5, "valid": 2044 x 2044
out_s2 = sysconv.sys_conv2d_strided(img, f, 2)            # every second row and column
torch.cuda.synchronize()
print("2-D:", tuple(out.shape), " stride 2:", tuple(out_s2.shape),
      " max |stride 2 - subsampled| =", float((out_s2 - out[::2, ::2]).abs().max()))
