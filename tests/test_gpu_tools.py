"""The diagnostic tools that ship with the library run end to end on the GPU."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_path_profile_tool():
    # the kernels compiled with the path profile (a library of its own, loaded in a process of its own):
    # every clock of the one replay of c1 is booked to a path, and the replay's results are what they are
    # without the marks
    res = subprocess.run([sys.executable, "-m", "paper_2503_20591_amd.path_profile", "c1"], cwd=ROOT, capture_output=True,
                         text=True, timeout=600)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "slowest replay (0)" in res.stdout and "rounds / immediate starts" in res.stdout
    import oracle
    from paper_2503_20591_amd import tracegen
    want = oracle.replay_batch(tracegen.workload("c1"))[0]
    assert f"'cells_started': {want['cells_started']}," in res.stdout
