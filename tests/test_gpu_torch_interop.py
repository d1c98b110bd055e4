"""PyTorch as the owner of device memory and streams (the paper's setting: a checkpoint engine under a
PyTorch training loop). Runs in a process of its own because PyTorch must be imported before the
library; everything else in this suite runs without PyTorch."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_snapshot_and_restore_of_torch_tensors():
    print("torch interop (subprocess)", flush=True)
    env = dict(os.environ, PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    r = subprocess.run([sys.executable, "-u", os.path.join(ROOT, "tests", "torch_interop_main.py")], capture_output=True, text=True,
                       timeout=420, cwd=ROOT, env=env)
    assert r.returncode == 0 and "torch interop ok" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
