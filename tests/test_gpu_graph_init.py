"""mecefo_init() prepares every kernel (dynamic-LDS limits, the static scratch address), so that the first
call of a process can already be recorded into a HIP graph: no eager warm-up call per shape is needed."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.mark.parametrize("tile", ["auto", "L8", "S"])
def test_first_call_of_a_fresh_process_under_graph_capture(tile):
    child = os.path.join(HERE, "graph_after_init_child.py")
    res = subprocess.run([sys.executable, "-u", child, tile], capture_output=True, text=True, timeout=110)
    assert res.returncode == 0, f"child failed ({res.returncode}):\n{res.stdout[-2000:]}\n{res.stderr[-4000:]}"
    assert res.stdout.strip().endswith("OK"), res.stdout[-2000:]
