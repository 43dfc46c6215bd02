"""The C ABI used from plain C: the example under paper_2605_12396_amd/examples compiles as C99 against include/nz.h
and libnz.so (CPU), and on a GPU it runs its checks (error bound after a roundtrip, exact doubling by the reduce)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2605_12396_amd")


def _build(tmp_path):
    exe = str(tmp_path / "roundtrip")
    cmd = ["gcc", "-std=c99", "-Wall", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
           os.path.join(PKG, "examples", "roundtrip.c"), "-L" + PKG, "-lnz", "-L/opt/rocm/lib", "-lamdhip64", "-lm",
           "-Wl,-rpath," + PKG, "-Wl,-rpath,/opt/rocm/lib", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


def test_example_compiles_as_c99(tmp_path):
    from paper_2605_12396_amd import binding
    binding.lib()                                   # (the library is built)
    assert os.path.exists(_build(tmp_path))


@pytest.mark.gpu
def test_example_runs(gpu_device, tmp_path):
    exe = _build(tmp_path)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "decodes to twice the values" in r.stdout
