"""The instrumented build of the library (same source, -DBT_TIMELINE): `bench.py --timeline` runs one cold
bt_compress and bt_decompress of configuration 2 with per-tile time stamps, checks that every tile's stamps
are in order and that the round trip is still bit exact, and prints the tables."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_timeline_mode_of_the_bench():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--timeline", "--sets", "4"],
                         capture_output=True, text=True, timeout=170, cwd=ROOT)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-2000:]
    assert "## bt_compress" in res.stdout and "## bt_decompress" in res.stdout
    assert res.stdout.count("Scanner passes that consumed counts") == 2
