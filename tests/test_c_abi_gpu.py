"""The C ABI driven from a plain C program (no Python, no PyTorch in the process): tests/c_abi_roundtrip.c."""
import os
import shutil
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
PKG = os.path.join(ROOT, "paper_1804_10223_amd")


def test_plain_c_program_rotates_a_permutation_bit_exactly(tmp_path):
    if shutil.which("gcc") is None or not os.path.exists("/opt/rocm/lib/libamdhip64.so"):
        pytest.skip("no C compiler or HIP runtime library here")
    exe = str(tmp_path / "c_abi_roundtrip")
    cmd = ["gcc", "-std=c99", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + os.path.join(ROOT, "include"),
           os.path.join(HERE, "c_abi_roundtrip.c"), "-o", exe, "-L" + PKG, "-l:libsprnn.so", "-L/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath," + PKG, "-Wl,-rpath,/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=100, env=dict(os.environ, SPRNN_DEBUG="1"))
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "0 mismatches" in r.stdout
