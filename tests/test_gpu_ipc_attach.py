"""Zero-copy attach of the weight pools from a second process (moe_pool_export / moe_pool_open; paper
Sec. 4.6 zero-copy, App. D): a memory-owner process exports its pools, a separate serving process opens
them, builds the layer over the attached memory and is graded against the oracle.  Both are fresh
processes started by a launcher that never touches the GPU (tests/ipc_roles.py); this test only starts
that launcher as a child process and reads its verdict."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu


def test_serving_process_runs_on_pools_owned_by_another_process():
    script = os.path.join(os.path.dirname(os.path.abspath(__file__)), "ipc_roles.py")
    r = subprocess.run([sys.executable, "-u", script, "launcher"], capture_output=True, text=True, timeout=600)
    print(r.stdout)
    print(r.stderr[-3000:])
    assert r.returncode == 0, f"launcher exit {r.returncode}"
    assert "forward max rel err" in r.stdout
