"""The C ABI from a plain C program: compiled with gcc against include/jsv.h, linked to
libjsv.so, run as a child process on the GPU."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plain_c_program(tmp_path):
    libdir = os.path.join(ROOT, "paper_2603_08797_amd")
    exe = str(tmp_path / "chain_demo")
    subprocess.check_call(["gcc", "-O1", "-Wall", "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c_abi", "chain_demo.c"),
                           "-L", libdir, "-ljsv", "-Wl,-rpath," + libdir, "-o", exe])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    sys.stdout.write(out.stdout)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "MISMATCH" not in out.stdout and out.stdout.count("ok") >= 9
