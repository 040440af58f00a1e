"""Launches longer than one grid dimension can hold are folded into (x, z).  That happens on
its own only beyond about 3e10 elements (tests/test_gpu_pipeline.py has one such compress);
here a child process lowers the fold point through the library's test variable and reruns
parity tests of every entry point with grids of 48 workgroups per row."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_kernel_with_a_folded_grid():
    env = dict(os.environ, TQ_TEST_MAX_GRID_X="48")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "gpu", "-p", "no:cacheprovider",
           "tests/test_gpu_pipeline.py::test_whole_path_matches_oracle",
           "tests/test_gpu_pipeline.py::test_whole_path_with_the_biscaled_codebook",
           "tests/test_gpu_update.py", "tests/test_gpu_simulate.py", "tests/test_gpu_multi.py",
           "tests/test_gpu_decode.py"]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-2000:]
