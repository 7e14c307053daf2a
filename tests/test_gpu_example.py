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


def test_c_abi_demo_runs():
    # plain C against include/dsk.h and the HIP runtime, built in-tree by `python -m paper_2411_02820_amd.build`
    exe = os.path.join(ROOT, "paper_2411_02820_amd", "dsk_c_demo")
    assert os.path.exists(exe), "dsk_c_demo is not built: run python -m paper_2411_02820_amd.build"
    r = subprocess.run([exe], capture_output=True, text=True, cwd=ROOT, timeout=120)
    print(r.stdout, r.stderr[-2000:])
    assert r.returncode == 0 and r.stdout.strip().endswith("ok")
