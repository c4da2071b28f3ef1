"""The C ABI from a caller that is not Python: tests/abi/abi_check (built by __graft_entry__.build() from
abi_check.cpp, the HIP runtime, libbitsnap.so and the C oracle) runs the four codecs and compares every output with
the oracle inside the same process."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BINARY = os.path.join(ROOT, "tests", "abi", "abi_check")


@pytest.mark.gpu
def test_c_program_through_the_abi():
    assert os.path.exists(BINARY), "tests/abi/abi_check is not built: run __graft_entry__.build()"
    print("[gpu-case] abi_check", flush=True)
    res = subprocess.run([BINARY], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "all checks passed" in res.stdout
