"""Launches longer than one grid dimension can hold are folded into (x, z).  That happens on
its own only beyond about 3e10 elements (tests/test_gpu_pipeline.py has one such compress);
here a child process loads the library's test build (the same sources with the fold point
adjustable), lowers the fold point and reruns parity tests of every entry point with grids of
48 workgroups per row."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_kernel_with_a_folded_grid():
    from paper_2402_01798_amd import build
    assert os.path.exists(build.FOLD_TEST_LIB), "build it first: python -m paper_2402_01798_amd.build"
    env = dict(os.environ, TQ_TEST_MAX_GRID_X="48", TQ_LIBRARY_PATH=build.FOLD_TEST_LIB)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "gpu", "-p", "no:cacheprovider",
           "tests/test_gpu_pipeline.py::test_whole_path_matches_oracle",
           "tests/test_gpu_pipeline.py::test_whole_path_with_the_biscaled_codebook",
           "tests/test_gpu_update.py", "tests/test_gpu_simulate.py", "tests/test_gpu_multi.py",
           "tests/test_gpu_decode.py"]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-2000:]
