"""The C-ABI library loads, exports every symbol include/tq.h declares, and rejects bad
arguments before touching a device (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tq.h")


@pytest.fixture(scope="module")
def L():
    from paper_2402_01798_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()                  # only when nothing is built; normally built beforehand
    return binding.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tq_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert set(names) == {"tq_num_buckets", "tq_payload_bytes", "tq_stats", "tq_stats_workspace_bytes", "tq_stats_static",
                          "tq_params",
                          "tq_compress", "tq_decompress_aggregate", "tq_decompress_aggregate_update",
                          "tq_quantize_dequantize", "tq_strerror",
                          "tq_stats_multi", "tq_params_multi", "tq_compress_multi",
                          "tq_stats_segments_workspace_bytes", "tq_stats_segments", "tq_compress_segments",
                          "tq_stats_segments_multi", "tq_compress_segments_multi",
                          "tq_decompress_aggregate_segments"}
    for n in names:
        assert getattr(L, n) is not None


def test_struct_sizes_match_the_oracle_side_layout():
    from oracle import binding as O
    from paper_2402_01798_amd import binding as B
    assert B.STATS_DTYPE.itemsize == O.STATS_DTYPE.itemsize == 3632
    assert B.PARAMS_DTYPE.itemsize == O.PARAMS_DTYPE.itemsize == 160
    assert B.STATS_DTYPE.fields.keys() == O.STATS_DTYPE.fields.keys()
    for k in B.PARAMS_DTYPE.fields:
        assert B.PARAMS_DTYPE.fields[k][1] == O.PARAMS_DTYPE.fields[k][1]
    for k in B.STATS_DTYPE.fields:
        assert B.STATS_DTYPE.fields[k][1] == O.STATS_DTYPE.fields[k][1]


def test_host_arithmetic(L):
    from oracle import binding as O
    for d, be in [(1, 0), (61706, 0), (1000, 384), (1 << 20, 1 << 20), (25_600_000, 1 << 20)]:
        assert L.tq_num_buckets(d, be) == O.num_buckets(d, be)
    for d in (1, 7, 8, 9, 127, 128, 61706, 11_200_000, 10 ** 9):
        for b in (2, 3, 4):
            assert L.tq_payload_bytes(d, b) == O.payload_bytes(d, b)
    assert L.tq_payload_bytes(61706, 3) == 23152


def test_bad_arguments_are_rejected_without_a_device(L):
    from paper_2402_01798_amd import binding as B
    p = C.c_void_p(0x1000)             # never dereferenced: every call below fails its checks
    odd = C.c_void_p(0x1004)
    assert L.tq_stats(p, 0, 0, 0, 0.0, p, p, 1 << 30, None) == B.EINVAL        # d = 0
    assert L.tq_stats(p, 7, 100, 0, 0.0, p, p, 1 << 30, None) == B.EINVAL      # dtype
    assert L.tq_stats(p, 0, 1000, 100, 0.0, p, p, 1 << 30, None) == B.EINVAL   # bucket not multiple of 128
    assert L.tq_stats(p, 0, 1000, 0, 1e-20, p, p, 1 << 30, None) == B.EINVAL   # g_min below the histogram
    assert L.tq_stats(odd, 0, 1000, 0, 0.0, p, p, 1 << 30, None) == B.EALIGN
    assert L.tq_stats(p, 0, 1000, 0, 0.0, p, p, 16, None) == B.EINVAL          # workspace too small
    assert L.tq_stats(p, 0, 1000, 0, 0.0, p, None, 1 << 30, None) == B.EINVAL  # no workspace
    assert L.tq_stats(None, 0, 1000, 0, 0.0, p, p, 1 << 30, None) == B.EINVAL
    assert L.tq_stats(p, 0, 1 << 32, 0, 0.0, p, p, 1 << 30, None) == B.EUNSUPPORTED    # 32-bit counts
    assert L.tq_stats(p, 0, 1 << 33, 1 << 32, 0.0, p, p, 1 << 30, None) == B.EUNSUPPORTED
    assert L.tq_params(p, 1, 5, 0, 0.0, p, None) == B.EINVAL                 # bits
    assert L.tq_params(p, 1, 3, 3, 0.0, p, None) == B.EINVAL                 # grid
    assert L.tq_params(p, 0, 3, 0, 0.0, p, None) == B.EINVAL                 # no buckets
    assert L.tq_params(p, 1, 3, 0, float("nan"), p, None) == B.EINVAL
    assert L.tq_compress(p, 0, 1000, 0, p, 1, 0, 0, 0, 0, p, None) == B.EINVAL  # bits
    assert L.tq_compress(p, 0, 1000, 0, p, 3, 7, 0, 0, 0, p, None) == B.EINVAL  # grid
    assert L.tq_compress(p, 0, 1000, 0, p, 3, 0, 0, 0, 0, odd, None) == B.EALIGN
    assert L.tq_compress(p, 0, 1 << 41, 0, p, 3, 1, 0, 0, 0, p, None) == B.EUNSUPPORTED
    arr = (C.c_void_p * 2)(0x1000, 0x2000)
    assert L.tq_decompress_aggregate(arr, arr, None, 0, 1000, 0, 3, 0, p, None) == B.EINVAL    # N = 0
    assert L.tq_decompress_aggregate(arr, arr, None, 65, 1000, 0, 3, 0, p, None) == B.EUNSUPPORTED
    assert L.tq_decompress_aggregate(arr, arr, None, 2, 1000, 0, 3, 0, odd, None) == B.EALIGN
    assert L.tq_quantize_dequantize(p, 0, 1000, 0, p, 6, 0, 0, 0, 0, p, None) == B.EINVAL     # bits
    assert L.tq_quantize_dequantize(p, 0, 1000, 0, p, 3, 0, 0, 0, 0, odd, None) == B.EALIGN
    assert L.tq_quantize_dequantize(p, 0, 1000, 0, None, 3, 0, 0, 0, 0, p, None) == B.EINVAL
    upd = L.tq_decompress_aggregate_update
    assert upd(arr, arr, None, 0, 1000, 0, 3, 0.1, 0.9, 0.0, p, None, None) == B.EINVAL      # N = 0
    assert upd(arr, arr, None, 2, 1000, 0, 5, 0.1, 0.9, 0.0, p, None, None) == B.EINVAL      # bits
    assert upd(arr, arr, None, 2, 1000, 0, 3, float("nan"), 0.9, 0.0, p, None, None) == B.EINVAL
    assert upd(arr, arr, None, 2, 1000, 0, 3, 0.1, 0.9, 0.0, None, None, None) == B.EINVAL   # no theta
    assert upd(arr, arr, None, 2, 1000, 0, 3, 0.1, 0.9, 0.0, p, p, None) == B.EINVAL         # velocity aliases theta
    assert upd(arr, arr, None, 2, 1000, 0, 3, 0.1, 0.9, 0.0, p, odd, None) == B.EALIGN
    bad = (C.c_void_p * 2)(0x1000, 0)
    assert L.tq_decompress_aggregate(bad, arr, None, 2, 1000, 0, 3, 0, p, None) == B.EINVAL    # null payload
    # the segment calls: the host copy of the table is checked before anything else
    import numpy as np
    good = np.array([0, 128, 1000], dtype=np.uint64)
    gp = good.ctypes.data_as(C.c_void_p)
    one = (C.c_void_p * 1)(0x1000)
    assert L.tq_stats_segments_multi(one, 0, 0, 1000, p, gp, 2, 0.0, one, p, 1 << 30, None) == B.EINVAL     # count = 0
    assert L.tq_stats_segments_multi(one, 65, 0, 1000, p, gp, 2, 0.0, one, p, 1 << 30, None) == B.EUNSUPPORTED
    assert L.tq_stats_segments_multi(one, 1, 0, 1000, p, gp, 2, 0.0, one, p, 16, None) == B.EINVAL         # workspace too small
    assert L.tq_stats_segments_multi(one, 1, 0, 1000, None, gp, 2, 0.0, one, p, 1 << 30, None) == B.EINVAL  # no device table
    bad = np.array([0, 100, 1000], dtype=np.uint64)                                # interior offset not a multiple of 128
    assert L.tq_stats_segments_multi(one, 1, 0, 1000, p, bad.ctypes.data_as(C.c_void_p), 2, 0.0, one, p, 1 << 30,
                                     None) == B.EINVAL
    big = np.array([0, 128, 1 << 32], dtype=np.uint64)                             # 32-bit counts
    assert L.tq_stats_segments_multi(one, 1, 0, 1 << 32, p, big.ctypes.data_as(C.c_void_p), 2, 0.0, one, p, 1 << 40,
                                     None) == B.EUNSUPPORTED
    assert L.tq_compress_segments_multi(one, 0, 0, 1000, p, gp, 2, one, 2, 0, 0, 0, one, None) == B.EINVAL   # count = 0
    assert L.tq_compress_segments_multi(one, 65, 0, 1000, p, gp, 2, one, 2, 0, 0, 0, one, None) == B.EUNSUPPORTED
    assert L.tq_compress_segments_multi(one, 1, 0, 1000, p, gp, 2, one, 5, 0, 0, 0, one, None) == B.EINVAL   # bits
    odd1 = (C.c_void_p * 1)(0x1004)
    assert L.tq_compress_segments_multi(odd1, 1, 0, 1000, p, gp, 2, one, 2, 0, 0, 0, one, None) == B.EALIGN
    assert L.tq_strerror(B.EALIGN).decode().startswith("device pointer")


def test_product_path_has_no_oracle_dependency():
    """The package must not import the oracle (it is test infrastructure)."""
    pkg = os.path.join(ROOT, "paper_2402_01798_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
