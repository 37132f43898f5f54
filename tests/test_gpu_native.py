"""The C ABI used without Python: tests/native/abi_smoke.bin (built by __graft_entry__.build())
allocates with hipMalloc, runs a refresh and a regular step through libgrass.so and compares
every result with the oracle library.  This test only runs it and reads its verdict."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
BIN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "abi_smoke.bin")


def test_stand_alone_c_abi_program_passes_its_own_parity_checks():
    assert os.path.exists(BIN), "build it with `python __graft_entry__.py` (or tests/native/build.py)"
    res = subprocess.run([BIN], capture_output=True, text=True, timeout=110)
    print(res.stdout)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "all checks passed" in res.stdout
    assert res.stdout.count(" ok ") >= 8
