"""The C ABI used from plain C (gcc, no Python, no torch): tests/c_abi/abi_check.c."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "abi_check")


def test_plain_c_caller_runs_the_whole_path():
    assert os.path.exists(EXE), "tests/c_abi/abi_check is not built: run python -m paper_2505_24179_amd.build"
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0 and "abi_check: ok" in r.stdout
