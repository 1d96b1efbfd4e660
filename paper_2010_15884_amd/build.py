"""Build libsysconv.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2010_15884_amd.build

hipcc cross-compiles without a GPU.  Packed-fp32 instructions are switched off
for the device pass (the kernels are written for v_fmac_f32 and its DPP form).
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsysconv.so")
SOURCES = ["api.hip", "conv1d.hip", "conv1d_arrays.hip", "conv1d_stride2.hip", "conv1d_stt.hip", "conv2d.hip", "conv2d_mfma.hip", "conv2d_stride2.hip", "copy.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# Per-file additions.  The matrix-core kernel keeps its accumulators in ordinary vector registers
# (the results go straight to the vector ALUs; from accumulation registers every value would
# first need a v_accvgpr_read).
FILE_FLAGS = {"conv2d_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    extra = os.environ.get("SYSCONV_EXTRA_FLAGS", "").split()      # build-time tunables (-DSYSCONV_...)
    cmd = ["hipcc", *FLAGS, *FILE_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True, lib: str = LIB) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    subprocess.run(cmd, check=True)
    if verbose:
        print(f"built {lib}")
    return lib


def build_c_demo(verbose: bool = True) -> str:
    """Compile examples/c_abi_demo.c with gcc as C99 against the built library: the
    header is plain C and the ABI needs nothing but the HIP runtime."""
    src = os.path.join(ROOT, "examples", "c_abi_demo.c")
    exe = os.path.join(ROOT, "examples", "c_abi_demo")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           "-I", os.path.join(ROOT, "include"), src, "-L", HERE, "-lsysconv", "-L/opt/rocm/lib", "-lamdhip64",
           "-lm", "-Wl,-rpath," + HERE, "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    subprocess.run(cmd, check=True)
    if verbose:
        print(f"built {exe}")
    return exe


SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
HOST_LOGIC = ["api.hip", "conv1d_stt.hip", "conv2d_mfma.hip"]      # argument checks, the design planner, the tap scaling


def build_host_sanitized(verbose: bool = True) -> str:
    """Host code of the library under AddressSanitizer + UndefinedBehaviorSanitizer (the device code is
    compiled as always): the translation units that hold host logic are rebuilt with the sanitizers on the
    host pass only, linked with the ordinary objects of the rest and with tests/abi_san_driver.cpp into an
    executable that needs no GPU."""
    san_dir = os.path.join(OBJ, "san")
    os.makedirs(san_dir, exist_ok=True)
    objs = []
    for src in SOURCES:
        if src in HOST_LOGIC:
            obj = os.path.join(san_dir, src.replace(".hip", ".o"))
            cmd = ["hipcc", *[f for f in FLAGS if f != "-O3"], "-O1", *SAN_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError(f"hipcc (host sanitizers) failed on {src}:\n{res.stderr}")
        else:
            obj = os.path.join(OBJ, src.replace(".hip", ".o"))
            if not os.path.exists(obj):
                _compile(src)
        objs.append(obj)
    exe = os.path.join(san_dir, "abi_san_driver")
    driver = os.path.join(ROOT, "tests", "abi_san_driver.cpp")
    cmd = ["hipcc", "--offload-arch=gfx950", "-std=c++17", "-O1", "-g", "-fsanitize=address", "-fsanitize=undefined",
           "-fno-sanitize-recover=all", "-fno-gpu-sanitize", "-I", os.path.join(ROOT, "include"), "-x", "c++", driver,
           "-x", "none", *objs, "-o", exe]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link of the sanitized host build failed:\n{res.stderr}")
    if verbose:
        print(f"built {exe}")
    return exe


if __name__ == "__main__":
    build()
    build_c_demo()
