"""Build libtq.so (HIP, gfx950) in-tree with hipcc.

Flags that are part of what the kernels mean:
  -ffp-contract=off   every binary32 operation on the element path is one IEEE rounding
                      (fused multiply-adds appear only where written, on exact products)
  -target-feature -packed-fp32-ops   no packed-fp32 instructions are generated
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtq.so")
# the same sources with the grid-fold test hook compiled in (tests/test_gpu_folded_grid.py only)
FOLD_TEST_LIB = os.path.join(HERE, "libtq_foldtest.so")

SOURCES = ["tq_api.hip", "tq_stats.hip", "tq_params.hip", "tq_compress.hip", "tq_decode.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wextra", "-Wno-unused-parameter",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _stale(out, deps):
    if not os.path.exists(out):
        return True
    t = os.path.getmtime(out)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, extra_flags=(), verbose: bool = False, lib: str = LIB, obj_dir: str = OBJ_DIR) -> str:
    """Compile every source to an object (in parallel) and link the shared library."""
    os.makedirs(obj_dir, exist_ok=True)
    headers = [os.path.join(ROOT, "include", "tq.h"), os.path.join(CSRC, "tq_device.h"),
               os.path.join(CSRC, "tq_layout.h"), __file__]

    def compile_one(src):
        s = os.path.join(CSRC, src)
        o = os.path.join(obj_dir, src.replace(".hip", ".o"))
        if force or _stale(o, [s] + headers):
            cmd = [HIPCC, *FLAGS, *extra_flags, "-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd))
            subprocess.check_call(cmd)
        return o

    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    if force or _stale(lib, objs):
        tmp = lib + ".tmp.%d" % os.getpid()
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
        os.replace(tmp, lib)
    return lib


def build_fold_test(force: bool = False, verbose: bool = False) -> str:
    """The test build: -DTQ_TEST_GRID_FOLD lets TQ_TEST_MAX_GRID_X lower the point at which long
    grids are folded, so that the folded path of every kernel can be driven with small inputs."""
    return build(force, ("-DTQ_TEST_GRID_FOLD",), verbose, FOLD_TEST_LIB, os.path.join(OBJ_DIR, "foldtest"))


if __name__ == "__main__":
    import sys
    print(build(force="--force" in sys.argv, verbose=True))
    print(build_fold_test(force="--force" in sys.argv, verbose=True))
