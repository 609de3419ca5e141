"""The C ABI used from a plain C program (tests/c_abi/spdnn_c_check.c, built by
__graft_entry__.build()): create, infer, introspection and an error path, checked
against the constant-row closed form of Eq. 1."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "c_abi", "spdnn_c_check")


@pytest.mark.gpu
def test_c_program_runs_the_library():
    assert os.path.exists(EXE), "build first: python __graft_entry__.py"
    lib_dir = os.path.join(ROOT, "paper_2007_14152_amd", "csrc")
    env = dict(os.environ, LD_LIBRARY_PATH=lib_dir + os.pathsep + os.environ.get("LD_LIBRARY_PATH", ""))
    out = subprocess.run([EXE], capture_output=True, text=True, timeout=100, env=env)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "c abi ok: 2 of 4 rows active" in out.stdout
