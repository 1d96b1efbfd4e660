"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only; nothing here touches a GPU).

Two legs: the CPU oracle (oracle/conv_oracle.c, driven by oracle/san_driver.c on exactly-sized heap buffers), and the
host side of libsysconv -- argument validation, the space-time-transform planner (Section 2.2's conditions) and the tap
scaling of the matrix-core path -- rebuilt with the sanitizers on the host pass only and driven by
tests/abi_san_driver.cpp with designs and sizes from the edges of what they accept.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(exe):
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=SAN_ENV)
    assert res.returncode == 0, f"{exe} failed:\n{res.stdout[-2000:]}\n{res.stderr[-4000:]}"
    assert "clean" in res.stdout
    assert "runtime error" not in res.stderr and "AddressSanitizer" not in res.stderr


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    if shutil.which("gcc") is None:
        pytest.skip("gcc is not installed")
    exe = str(tmp_path / "oracle_san_driver")
    cmd = ["gcc", "-std=c99", "-g", "-O1", "-fopenmp", "-Wall", "-Wextra", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan",
           os.path.join(ROOT, "oracle", "conv_oracle.c"), os.path.join(ROOT, "oracle", "san_driver.c"), "-lm", "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    _run(exe)


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers():
    if shutil.which("hipcc") is None:
        pytest.skip("hipcc is not installed")
    from paper_2010_15884_amd import build
    _run(build.build_host_sanitized(verbose=False))
