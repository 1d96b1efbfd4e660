"""The boundary is a C ABI: a C99 program built with gcc (no C++, no Python, no torch)
uses it through include/sysconv.h."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "examples", "c_abi_demo")


def test_header_and_demo_compile_as_c99_with_gcc():
    from paper_2010_15884_amd import build
    if not os.path.exists(build.LIB):
        pytest.skip("libsysconv.so is not built")
    exe = build.build_c_demo(verbose=False)
    assert os.path.exists(exe)


@pytest.mark.gpu
def test_c_demo_runs_on_the_gpu():
    if not os.path.exists(EXE):
        from paper_2010_15884_amd import build
        build.build_c_demo(verbose=False)
    res = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(res.stdout)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "all good" in res.stdout
