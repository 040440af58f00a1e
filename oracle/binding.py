"""ctypes front end of ``tq_oracle.c`` -- TEST INFRASTRUCTURE (see that file's header).

All arrays are host numpy arrays.  ``stats`` and ``params`` travel as numpy
structured arrays whose dtypes mirror the C structs byte for byte, so a test
can hand the very same bytes to the GPU library.
"""
import ctypes as C

import numpy as np

from . import build as _build

NBINS = 898
F32, BF16 = 0, 1
GRID_UNIFORM, GRID_NONUNIFORM, GRID_BISCALED = 0, 1, 2

STATS_DTYPE = np.dtype([
    ("hist", np.uint32, (NBINS,)),
    ("n_nonfinite", np.uint32),
    ("absmax", np.float32),
    ("n", np.uint64),
    ("g_min", np.float32),
    ("reserved", np.uint32),
    ("n_tail", np.uint64),
    ("sum_log_tail", np.float64),
], align=True)

PARAMS_DTYPE = np.dtype([
    ("alpha", np.float32),
    ("bits", np.uint32),
    ("s", np.uint32),
    ("grid", np.uint32),
    ("level", np.float32, (16,)),
    ("inv_w", np.float32, (16,)),
    ("gamma_hat", np.float32),
    ("rho_hat", np.float32),
    ("g_min", np.float32),
    ("flags", np.uint32),
], align=True)

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        L.tqo_philox4x32.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.tqo_philox4x32.restype = None
        L.tqo_rand16.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64]
        L.tqo_rand16.restype = C.c_uint32
        L.tqo_truncate.argtypes = [C.c_float, C.c_float]
        L.tqo_truncate.restype = C.c_float
        L.tqo_quantize_one.argtypes = [C.c_float, C.c_void_p, C.c_uint32]
        L.tqo_quantize_one.restype = C.c_uint32
        L.tqo_quantize_eq2.argtypes = [C.c_float, C.c_void_p, C.c_uint32]
        L.tqo_quantize_eq2.restype = C.c_uint32
        L.tqo_enumerate_draws.argtypes = [C.c_float, C.c_void_p, C.c_int, C.c_void_p]
        L.tqo_enumerate_draws.restype = None
        L.tqo_bin.argtypes = [C.c_float]
        L.tqo_bin.restype = C.c_uint32
        L.tqo_num_buckets.argtypes = [C.c_uint64, C.c_uint64]
        L.tqo_num_buckets.restype = C.c_uint64
        L.tqo_payload_bytes.argtypes = [C.c_uint64, C.c_int]
        L.tqo_payload_bytes.restype = C.c_uint64
        L.tqo_stats.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_uint64,
                                C.c_float, C.c_void_p]
        L.tqo_stats_buckets.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_uint64,
                                        C.c_float, C.c_void_p, C.c_uint64, C.c_uint64]
        L.tqo_compress.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_uint64,
                                   C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32,
                                   C.c_void_p]
        L.tqo_compress_range.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_uint64,
                                         C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32,
                                         C.c_void_p, C.c_uint64, C.c_uint64]
        L.tqo_decompress_aggregate_range.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p,
                                                     C.c_int, C.c_uint64, C.c_uint64,
                                                     C.c_int, C.c_int, C.c_void_p,
                                                     C.c_uint64, C.c_uint64]
        L.tqo_decompress_aggregate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_int, C.c_uint64, C.c_uint64,
                                               C.c_int, C.c_int, C.c_void_p]
        L.tqo_decompress_aggregate_update.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p,
                                                      C.c_int, C.c_uint64, C.c_uint64, C.c_int,
                                                      C.c_float, C.c_float, C.c_float,
                                                      C.c_void_p, C.c_void_p]
        L.tqo_dequantize.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64,
                                     C.c_int, C.c_void_p]
        L.tqo_stats_segments.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_void_p, C.c_uint64,
                                         C.c_float, C.c_void_p]
        L.tqo_compress_segments.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_void_p, C.c_uint64,
                                            C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32, C.c_void_p]
        L.tqo_decompress_aggregate_segments.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int,
                                                        C.c_uint64, C.c_void_p, C.c_uint64, C.c_int,
                                                        C.c_int, C.c_void_p]
        L.tqo_sizeof_stats.restype = C.c_size_t
        L.tqo_sizeof_params.restype = C.c_size_t
        assert L.tqo_sizeof_stats() == STATS_DTYPE.itemsize
        assert L.tqo_sizeof_params() == PARAMS_DTYPE.itemsize
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _dtype_code(g):
    if g.dtype == np.float32:
        return F32
    if g.dtype == np.uint16:      # bf16 bit patterns
        return BF16
    raise TypeError("gradient must be float32 or uint16 (bf16 bits), got %s" % g.dtype)


def _check(rc, what):
    if rc != 0:
        raise ValueError("%s rejected its arguments (code %d)" % (what, rc))


def philox4x32(ctr, key, rounds=10):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().tqo_philox4x32(_ptr(c), _ptr(k), rounds, _ptr(out))
    return out


def rand16(seed, worker, step, e):
    return int(lib().tqo_rand16(seed, worker, step, e))


def truncate(g, alpha):
    return float(lib().tqo_truncate(g, alpha))


def quantize_one(g, params, r):
    """Code chosen for the scalar ``g`` under one ``PARAMS_DTYPE`` record and draw ``r``."""
    p = np.ascontiguousarray(params).reshape(-1)[:1]
    return int(lib().tqo_quantize_one(float(g), _ptr(p), int(r)))


def quantize_eq2(g, params, r):
    """Eq. (2) step by step (cell by comparison, p_r, the draw): the definition."""
    p = np.ascontiguousarray(params).reshape(-1)[:1]
    return int(lib().tqo_quantize_eq2(float(g), _ptr(p), int(r)))


def enumerate_draws(g, params, eq2=False):
    """count[c] = how many of the 65,536 draws give code c for the value ``g``."""
    p = np.ascontiguousarray(params).reshape(-1)[:1]
    out = np.zeros(16, dtype=np.uint32)
    lib().tqo_enumerate_draws(float(g), _ptr(p), int(bool(eq2)), _ptr(out))
    return out


def _run_ranges(n_items, threads, align, call):
    """``call(lo, hi)`` over [0, n_items) cut into ``threads`` ranges whose starts are
    multiples of ``align``; on host threads when threads > 1 (ctypes drops the GIL)."""
    threads = max(1, int(threads))
    if threads == 1 or n_items <= align:
        return [call(0, n_items)]
    per = -(-n_items // threads)
    per = -(-per // align) * align
    cuts = [(lo, min(lo + per, n_items)) for lo in range(0, n_items, per)]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda c: call(*c), cuts))


def bin_index(a):
    return int(lib().tqo_bin(float(a)))


def num_buckets(d, bucket_elems):
    return int(lib().tqo_num_buckets(d, bucket_elems))


def payload_bytes(d, bits):
    return int(lib().tqo_payload_bytes(d, bits))


def stats(g, bucket_elems=0, g_min=0.0, threads=1):
    """Per-bucket statistics; ``threads`` > 1 spreads the buckets over host threads."""
    g = np.ascontiguousarray(g)
    nb = num_buckets(g.size, bucket_elems)
    out = np.zeros(nb, dtype=STATS_DTYPE)
    L, code = lib(), _dtype_code(g)
    rcs = _run_ranges(nb, threads, 1, lambda lo, hi: L.tqo_stats_buckets(
        _ptr(g), code, g.size, bucket_elems, float(g_min), _ptr(out), lo, hi))
    for rc in rcs:
        _check(rc, "tqo_stats")
    return out


def compress(g, params, seed, worker, step, bucket_elems=0, threads=1):
    """One worker's payload; ``threads`` > 1 encodes disjoint element ranges on host threads."""
    g = np.ascontiguousarray(g)
    params = np.ascontiguousarray(params, dtype=PARAMS_DTYPE).reshape(-1)
    assert params.size == num_buckets(g.size, bucket_elems)
    bits = int(params["bits"][0])
    out = np.zeros(payload_bytes(g.size, bits), dtype=np.uint8)
    L, code = lib(), _dtype_code(g)
    rcs = _run_ranges(g.size, threads, 4096, lambda lo, hi: L.tqo_compress_range(
        _ptr(g), code, g.size, bucket_elems, _ptr(params), seed, worker, step, _ptr(out), lo, hi))
    for rc in rcs:
        _check(rc, "tqo_compress")
    return out


def decompress_aggregate(payloads, params, d, bits, bucket_elems=0, weights=None,
                         out=None, threads=1):
    """``payloads``/``params``: one array per worker.  ``out`` given => accumulate into it."""
    N = len(payloads)
    payloads = [np.ascontiguousarray(p, dtype=np.uint8) for p in payloads]
    params = [np.ascontiguousarray(p, dtype=PARAMS_DTYPE).reshape(-1) for p in params]
    pp = (C.c_void_p * N)(*[p.ctypes.data for p in payloads])
    qq = (C.c_void_p * N)(*[p.ctypes.data for p in params])
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
    accumulate = out is not None
    if out is None:
        out = np.zeros(d, dtype=np.float32)
    L = lib()
    rcs = _run_ranges(d, threads, 4096, lambda lo, hi: L.tqo_decompress_aggregate_range(
        pp, qq, None if w is None else _ptr(w), N, d, bucket_elems, bits, int(accumulate),
        _ptr(out), lo, hi))
    for rc in rcs:
        _check(rc, "tqo_decompress_aggregate")
    return out


def decompress_aggregate_update(payloads, params, theta, bits, eta, momentum=0.0,
                                weight_decay=0.0, velocity=None, bucket_elems=0, weights=None):
    """Alg. 1's two server steps in place on ``theta`` (and ``velocity`` when given), float32."""
    N = len(payloads)
    assert theta.dtype == np.float32 and theta.flags.c_contiguous
    assert velocity is None or (velocity.dtype == np.float32 and velocity.flags.c_contiguous
                                and velocity.size == theta.size)
    payloads = [np.ascontiguousarray(p, dtype=np.uint8) for p in payloads]
    params = [np.ascontiguousarray(p, dtype=PARAMS_DTYPE).reshape(-1) for p in params]
    pp = (C.c_void_p * N)(*[p.ctypes.data for p in payloads])
    qq = (C.c_void_p * N)(*[p.ctypes.data for p in params])
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
    _check(lib().tqo_decompress_aggregate_update(
        pp, qq, None if w is None else _ptr(w), N, theta.size, bucket_elems, bits, eta, momentum,
        weight_decay, _ptr(theta), None if velocity is None else _ptr(velocity)),
        "tqo_decompress_aggregate_update")
    return theta


def quantize_dequantize(g, params, seed, worker, step, bucket_elems=0):
    """Q[T_alpha(g)] as values: the client step of Alg. 1 followed by the server's look-up."""
    params = np.ascontiguousarray(params, dtype=PARAMS_DTYPE).reshape(-1)
    bits = int(params["bits"][0])
    return dequantize(compress(g, params, seed, worker, step, bucket_elems=bucket_elems), params, g.size, bits,
                      bucket_elems=bucket_elems)


def dequantize(payload, params, d, bits, bucket_elems=0):
    payload = np.ascontiguousarray(payload, dtype=np.uint8)
    params = np.ascontiguousarray(params, dtype=PARAMS_DTYPE).reshape(-1)
    out = np.zeros(d, dtype=np.float32)
    _check(lib().tqo_dequantize(_ptr(payload), _ptr(params), d, bucket_elems, bits,
                                _ptr(out)), "tqo_dequantize")
    return out


def _offsets(seg_offsets, d):
    off = np.ascontiguousarray(seg_offsets, dtype=np.uint64)
    assert off.ndim == 1 and off.size >= 2 and int(off[-1]) == d
    return off


def stats_segments(g, seg_offsets, g_min=0.0):
    """One STATS_DTYPE record per segment [seg_offsets[s], seg_offsets[s+1])."""
    g = np.ascontiguousarray(g)
    off = _offsets(seg_offsets, g.size)
    out = np.zeros(off.size - 1, dtype=STATS_DTYPE)
    _check(lib().tqo_stats_segments(_ptr(g), _dtype_code(g), g.size, _ptr(off), off.size - 1,
                                    float(g_min), _ptr(out)), "tqo_stats_segments")
    return out


def compress_segments(g, seg_offsets, params, seed, worker, step):
    g = np.ascontiguousarray(g)
    off = _offsets(seg_offsets, g.size)
    params = np.ascontiguousarray(params, dtype=PARAMS_DTYPE).reshape(-1)
    assert params.size == off.size - 1
    bits = int(params["bits"][0])
    out = np.zeros(payload_bytes(g.size, bits), dtype=np.uint8)
    _check(lib().tqo_compress_segments(_ptr(g), _dtype_code(g), g.size, _ptr(off), off.size - 1,
                                       _ptr(params), seed, worker, step, _ptr(out)),
           "tqo_compress_segments")
    return out


def decompress_aggregate_segments(payloads, params, d, seg_offsets, bits, weights=None, out=None):
    N = len(payloads)
    off = _offsets(seg_offsets, d)
    payloads = [np.ascontiguousarray(p, dtype=np.uint8) for p in payloads]
    params = [np.ascontiguousarray(p, dtype=PARAMS_DTYPE).reshape(-1) for p in params]
    pp = (C.c_void_p * N)(*[p.ctypes.data for p in payloads])
    qq = (C.c_void_p * N)(*[p.ctypes.data for p in params])
    w = None if weights is None else np.ascontiguousarray(weights, dtype=np.float32)
    accumulate = out is not None
    if out is None:
        out = np.zeros(d, dtype=np.float32)
    _check(lib().tqo_decompress_aggregate_segments(pp, qq, None if w is None else _ptr(w), N, d,
                                                   _ptr(off), off.size - 1, bits, int(accumulate),
                                                   _ptr(out)), "tqo_decompress_aggregate_segments")
    return out
