"""Helpers of the GPU parity tests: run the HIP path through the C ABI and
compare it with the CPU oracle, output by output.

Tolerance: max_i |y_gpu[i] - y_ref[i]| / sum_k |w[k]||x[i+k]|  <=  1e-5.
An fp32 chain of K fused or unfused multiply-adds in any order errs by at most
about K * 2^-24 of that scale (K = 121 gives 7.2e-6), so every projection and
summation order passes and a dropped or misplaced tap does not.
"""
import numpy as np
import torch

import oracle
from paper_2010_15884_amd import binding as B

TOL = 1e-5
ORACLE_THREADS = 16


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run1d(x, w, proj):
    y = B.sys_conv1d(dev(x), w, projection=proj)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def run2d(x, f, proj):
    y = B.sys_conv2d(dev(x), f, projection=proj)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def err1d(y, x, w):
    ref = oracle.conv1d(x, w, ORACLE_THREADS)
    scale = oracle.absdot1d(x, w, ORACLE_THREADS)
    return oracle.max_rel_err(y, ref, scale)


def err2d(y, x, f):
    ref = oracle.conv2d(x, f, ORACLE_THREADS)
    scale = oracle.absdot2d(x, f, ORACLE_THREADS)
    return oracle.max_rel_err(y, ref, scale)
