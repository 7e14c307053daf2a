"""The end-to-end example (store, fetch, selective prefill, suffix; Sec. 4.4) runs and reports success."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_selective_prefill_example_runs():
    r = subprocess.run([sys.executable, "-m", "paper_2411_02820_amd.examples.selective_prefill"], capture_output=True,
                       text=True, cwd=ROOT, timeout=300)
    print(r.stdout, r.stderr[-2000:])
    assert r.returncode == 0 and r.stdout.strip().endswith("ok")
