"""The C ABI from plain C: tests/c_client/roundtrip (built by __graft_entry__.build() with gcc) allocates
with the HIP runtime, calls libbittrain.so and checks every output against the C oracle linked into it."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_client", "roundtrip")


def test_c_program_round_trip():
    if not os.path.exists(EXE):
        pytest.fail("tests/c_client/roundtrip is not built: run __graft_entry__.build()")
    res = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "c_client ok" in res.stdout
    assert res.stdout.count(" ok\n") == 7 and "MISMATCH" not in res.stdout      # six cases and the summary line
