"""Thin ctypes layer over ``libtq.so``: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used purely as device memory; every call passes
``data_ptr()`` values and the current HIP stream to the library.  There is no fallback:
if the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# TQ_LIBRARY_PATH selects another build of the same library (the tests' grid-fold build)
LIB_PATH = os.environ.get("TQ_LIBRARY_PATH") or os.path.join(HERE, "libtq.so")

OK, EINVAL, EALIGN, EUNSUPPORTED, EHIP = 0, 1, 2, 3, 4
F32, BF16 = 0, 1
GRID_UNIFORM, GRID_NONUNIFORM, GRID_BISCALED = 0, 1, 2
NBINS = 898
MAX_WORKERS = 64
STATS_BYTES = 3632
PARAMS_BYTES = 160

# numpy views of the interface structs (layout fixed by include/tq.h)
STATS_DTYPE = np.dtype([
    ("hist", np.uint32, (NBINS,)), ("n_nonfinite", np.uint32), ("absmax", np.float32),
    ("n", np.uint64), ("g_min", np.float32), ("reserved", np.uint32),
    ("n_tail", np.uint64), ("sum_log_tail", np.float64)], align=True)
PARAMS_DTYPE = np.dtype([
    ("alpha", np.float32), ("bits", np.uint32), ("s", np.uint32), ("grid", np.uint32),
    ("level", np.float32, (16,)), ("inv_w", np.float32, (16,)),
    ("gamma_hat", np.float32), ("rho_hat", np.float32), ("g_min", np.float32),
    ("flags", np.uint32)], align=True)
assert STATS_DTYPE.itemsize == STATS_BYTES and PARAMS_DTYPE.itemsize == PARAMS_BYTES


class TqError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s: %s (code %d)" % (what, strerror(code), code))


_lib = None


def lib():
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: build it with `python -m paper_2402_01798_amd.build`" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        u64, u32, i32, f32, vp = C.c_uint64, C.c_uint32, C.c_int, C.c_float, C.c_void_p
        L.tq_num_buckets.argtypes = [u64, u64]
        L.tq_num_buckets.restype = u64
        L.tq_payload_bytes.argtypes = [u64, i32]
        L.tq_payload_bytes.restype = u64
        L.tq_stats_workspace_bytes.argtypes = [u64, u64]
        L.tq_stats_workspace_bytes.restype = u64
        L.tq_stats.argtypes = [vp, i32, u64, u64, f32, vp, vp, u64, vp]
        L.tq_stats_static.argtypes = [vp, i32, u64, u64, f32, vp, vp]
        L.tq_params.argtypes = [vp, u64, i32, i32, f32, vp, vp]
        L.tq_compress.argtypes = [vp, i32, u64, u64, vp, i32, i32, u64, u32, u32, vp, vp]
        L.tq_decompress_aggregate.argtypes = [vp, vp, vp, i32, u64, u64, i32, i32, vp, vp]
        L.tq_decompress_aggregate_update.argtypes = [vp, vp, vp, i32, u64, u64, i32, f32, f32, f32, vp, vp, vp]
        L.tq_quantize_dequantize.argtypes = [vp, i32, u64, u64, vp, i32, u64, u32, u32, i32, vp, vp]
        L.tq_quantize_dequantize.restype = i32
        L.tq_strerror.argtypes = [i32]
        L.tq_strerror.restype = C.c_char_p
        L.tq_stats_multi.argtypes = [vp, i32, i32, u64, u64, f32, vp, vp, u64, vp]
        L.tq_params_multi.argtypes = [vp, i32, u64, i32, i32, f32, vp, vp]
        L.tq_compress_multi.argtypes = [vp, i32, i32, u64, u64, vp, i32, i32, u64, u32, u32, vp, vp]
        L.tq_stats_segments_workspace_bytes.argtypes = [u64, u64]
        L.tq_stats_segments_workspace_bytes.restype = u64
        L.tq_stats_segments.argtypes = [vp, i32, u64, vp, vp, u64, f32, vp, vp, u64, vp]
        L.tq_compress_segments.argtypes = [vp, i32, u64, vp, vp, u64, vp, i32, u64, u32, u32, vp, vp]
        L.tq_decompress_aggregate_segments.argtypes = [vp, vp, vp, i32, u64, vp, vp, u64, i32, i32, vp, vp]
        L.tq_stats_segments_multi.argtypes = [vp, i32, i32, u64, vp, vp, u64, f32, vp, vp, u64, vp]
        L.tq_compress_segments_multi.argtypes = [vp, i32, i32, u64, vp, vp, u64, vp, i32, u64, u32, u32, vp, vp]
        for f in (L.tq_stats_segments, L.tq_compress_segments, L.tq_decompress_aggregate_segments,
                  L.tq_stats_segments_multi, L.tq_compress_segments_multi):
            f.restype = i32
        for f in (L.tq_stats, L.tq_stats_static, L.tq_params, L.tq_compress, L.tq_decompress_aggregate,
                  L.tq_decompress_aggregate_update, L.tq_stats_multi, L.tq_params_multi, L.tq_compress_multi):
            f.restype = i32
        _lib = L
    return _lib


def strerror(code):
    return lib().tq_strerror(code).decode()


def _check(rc, what):
    if rc != OK:
        raise TqError(rc, what)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(g):
    if g.dtype == torch.float32:
        return F32
    if g.dtype == torch.bfloat16:
        return BF16
    raise TypeError("gradient must be float32 or bfloat16, got %s" % g.dtype)


def _dev(t, what):
    if not (t.is_cuda and t.is_contiguous()):
        raise ValueError("%s must be a contiguous device tensor" % what)
    return C.c_void_p(t.data_ptr())


def num_buckets(d, bucket_elems=0):
    return int(lib().tq_num_buckets(d, bucket_elems))


def payload_bytes(d, bits):
    return int(lib().tq_payload_bytes(d, bits))


def alloc_stats(d, bucket_elems=0, device="cuda"):
    return torch.empty(num_buckets(d, bucket_elems) * STATS_BYTES, dtype=torch.uint8, device=device)


def stats_workspace_bytes(d, bucket_elems=0):
    return int(lib().tq_stats_workspace_bytes(d, bucket_elems))


def alloc_stats_workspace(d, bucket_elems=0, device="cuda"):
    return torch.empty(stats_workspace_bytes(d, bucket_elems), dtype=torch.uint8, device=device)


def alloc_params(d, bucket_elems=0, device="cuda"):
    return torch.empty(num_buckets(d, bucket_elems) * PARAMS_BYTES, dtype=torch.uint8, device=device)


def alloc_payload(d, bits, device="cuda"):
    return torch.empty(payload_bytes(d, bits), dtype=torch.uint8, device=device)


def tq_stats(g, stats, workspace, bucket_elems=0, g_min=0.0):
    _check(lib().tq_stats(_dev(g, "g"), _dtype_code(g), g.numel(), bucket_elems, g_min,
                          _dev(stats, "stats"), _dev(workspace, "workspace"), workspace.numel(),
                          _stream()), "tq_stats")
    return stats


def tq_stats_static(g, stats, bucket_elems=0, g_min=0.0):
    _check(lib().tq_stats_static(_dev(g, "g"), _dtype_code(g), g.numel(), bucket_elems, g_min,
                                 _dev(stats, "stats"), _stream()), "tq_stats_static")
    return stats


def tq_params(stats, params, bits, grid, alpha_override=0.0):
    nb = stats.numel() // STATS_BYTES
    if params.numel() != nb * PARAMS_BYTES:
        raise ValueError("params buffer does not match the number of buckets")
    _check(lib().tq_params(_dev(stats, "stats"), nb, bits, grid, alpha_override,
                           _dev(params, "params"), _stream()), "tq_params")
    return params


def tq_compress(g, params, payload, bits, seed, worker, step, bucket_elems=0, grid=GRID_UNIFORM):
    """``grid``: the family ``params`` was designed with; it only shapes the launch (see tq.h)."""
    d = g.numel()
    if params.numel() != num_buckets(d, bucket_elems) * PARAMS_BYTES:
        raise ValueError("params buffer does not match the number of buckets")
    if payload.numel() < payload_bytes(d, bits):
        raise ValueError("payload buffer too small")
    _check(lib().tq_compress(_dev(g, "g"), _dtype_code(g), d, bucket_elems, _dev(params, "params"),
                             bits, grid, seed, worker, step, _dev(payload, "payload"), _stream()),
           "tq_compress")
    return payload


def tq_quantize_dequantize(g, params, out, bits, seed, worker, step, bucket_elems=0, accumulate=False):
    d = g.numel()
    if params.numel() != num_buckets(d, bucket_elems) * PARAMS_BYTES:
        raise ValueError("params buffer does not match the number of buckets")
    if out.dtype != torch.float32 or out.numel() != d:
        raise ValueError("out must be float32 of the gradient's size")
    _check(lib().tq_quantize_dequantize(_dev(g, "g"), _dtype_code(g), d, bucket_elems, _dev(params, "params"),
                                        bits, seed, worker, step, int(bool(accumulate)), _dev(out, "out"),
                                        _stream()), "tq_quantize_dequantize")
    return out


def _ptr_array(tensors, what):
    return (C.c_void_p * len(tensors))(*[_dev(t, what).value for t in tensors])


def tq_stats_multi(gs, stats, workspace, bucket_elems=0, g_min=0.0):
    """Batched tq_stats: lists of same-shaped gradients and their stats buffers."""
    _check(lib().tq_stats_multi(_ptr_array(gs, "g"), len(gs), _dtype_code(gs[0]), gs[0].numel(),
                                bucket_elems, g_min, _ptr_array(stats, "stats"),
                                _dev(workspace, "workspace"), workspace.numel(), _stream()),
           "tq_stats_multi")
    return stats


def tq_params_multi(stats, params, bits, grid, alpha_override=0.0):
    nb = stats[0].numel() // STATS_BYTES
    _check(lib().tq_params_multi(_ptr_array(stats, "stats"), len(stats), nb, bits, grid, alpha_override,
                                 _ptr_array(params, "params"), _stream()), "tq_params_multi")
    return params


def tq_compress_multi(gs, params, payloads, bits, seed, first_worker, step, bucket_elems=0, grid=GRID_UNIFORM):
    d = gs[0].numel()
    for g, q, p in zip(gs, params, payloads):
        if g.numel() != d or g.dtype != gs[0].dtype:
            raise ValueError("batched tensors must share shape and dtype")
        if q.numel() != num_buckets(d, bucket_elems) * PARAMS_BYTES or p.numel() < payload_bytes(d, bits):
            raise ValueError("params / payload buffer size does not match d")
    _check(lib().tq_compress_multi(_ptr_array(gs, "g"), len(gs), _dtype_code(gs[0]), d, bucket_elems,
                                   _ptr_array(params, "params"), bits, grid, seed, first_worker, step,
                                   _ptr_array(payloads, "payload"), _stream()), "tq_compress_multi")
    return payloads


def _decode_args(payloads, params, d, bits, bucket_elems, weights):
    N = len(payloads)
    if len(params) != N:
        raise ValueError("one params buffer per payload")
    nb = num_buckets(d, bucket_elems)
    for p, q in zip(payloads, params):
        if p.numel() < payload_bytes(d, bits) or q.numel() != nb * PARAMS_BYTES:
            raise ValueError("payload / params buffer size does not match d")
    pp = (C.c_void_p * N)(*[_dev(p, "payload").value for p in payloads])
    qq = (C.c_void_p * N)(*[_dev(q, "params").value for q in params])
    ww = None
    if weights is not None:
        if len(weights) != N:
            raise ValueError("one weight per worker")
        ww = (C.c_float * N)(*[float(w) for w in weights])
    return pp, qq, ww, N


def tq_decompress_aggregate(payloads, params, out, bits, bucket_elems=0, weights=None,
                            accumulate=False):
    d = out.numel()
    if out.dtype != torch.float32:
        raise TypeError("out must be float32")
    pp, qq, ww, N = _decode_args(payloads, params, d, bits, bucket_elems, weights)
    _check(lib().tq_decompress_aggregate(pp, qq, ww, N, d, bucket_elems, bits, int(bool(accumulate)),
                                         _dev(out, "out"), _stream()), "tq_decompress_aggregate")
    return out


def tq_decompress_aggregate_update(payloads, params, theta, bits, eta, momentum=0.0, weight_decay=0.0,
                                   velocity=None, bucket_elems=0, weights=None):
    d = theta.numel()
    if theta.dtype != torch.float32 or (velocity is not None and velocity.dtype != torch.float32):
        raise TypeError("theta and velocity must be float32")
    if velocity is not None and velocity.numel() != d:
        raise ValueError("velocity must have theta's size")
    pp, qq, ww, N = _decode_args(payloads, params, d, bits, bucket_elems, weights)
    _check(lib().tq_decompress_aggregate_update(
        pp, qq, ww, N, d, bucket_elems, bits, float(eta), float(momentum), float(weight_decay),
        _dev(theta, "theta"), None if velocity is None else _dev(velocity, "velocity"), _stream()),
        "tq_decompress_aggregate_update")
    return theta


class Segments:
    """A segment table in both memories: ``offsets`` (host, numpy uint64, nseg + 1 entries) and
    its device copy.  Pure marshalling: the library checks the host copy."""

    def __init__(self, offsets, device="cuda"):
        self.host = np.ascontiguousarray(offsets, dtype=np.uint64)
        self.dev = torch.from_numpy(self.host.view(np.int64).copy()).to(device)
        self.nseg = self.host.size - 1
        self.d = int(self.host[-1])

    def args(self):
        return C.c_void_p(self.dev.data_ptr()), self.host.ctypes.data_as(C.c_void_p), self.nseg


def stats_segments_workspace_bytes(d, nseg):
    return int(lib().tq_stats_segments_workspace_bytes(d, nseg))


def tq_stats_segments(g, seg, stats, workspace, g_min=0.0):
    dev, host, nseg = seg.args()
    _check(lib().tq_stats_segments(_dev(g, "g"), _dtype_code(g), g.numel(), dev, host, nseg, g_min,
                                   _dev(stats, "stats"), _dev(workspace, "workspace"), workspace.numel(),
                                   _stream()), "tq_stats_segments")
    return stats


def tq_compress_segments(g, seg, params, payload, bits, seed, worker, step):
    d = g.numel()
    if params.numel() != seg.nseg * PARAMS_BYTES or payload.numel() < payload_bytes(d, bits):
        raise ValueError("params / payload buffer size does not match the segments")
    dev, host, nseg = seg.args()
    _check(lib().tq_compress_segments(_dev(g, "g"), _dtype_code(g), d, dev, host, nseg, _dev(params, "params"),
                                      bits, seed, worker, step, _dev(payload, "payload"), _stream()),
           "tq_compress_segments")
    return payload


def tq_stats_segments_multi(gs, seg, stats, workspace, g_min=0.0):
    """Batched tq_stats_segments: same-shaped gradients that share the segment table."""
    dev, host, nseg = seg.args()
    _check(lib().tq_stats_segments_multi(_ptr_array(gs, "g"), len(gs), _dtype_code(gs[0]), gs[0].numel(), dev, host,
                                         nseg, g_min, _ptr_array(stats, "stats"), _dev(workspace, "workspace"),
                                         workspace.numel(), _stream()), "tq_stats_segments_multi")
    return stats


def tq_compress_segments_multi(gs, seg, params, payloads, bits, seed, first_worker, step):
    d = gs[0].numel()
    for g, q, p in zip(gs, params, payloads):
        if g.numel() != d or g.dtype != gs[0].dtype:
            raise ValueError("batched tensors must share shape and dtype")
        if q.numel() != seg.nseg * PARAMS_BYTES or p.numel() < payload_bytes(d, bits):
            raise ValueError("params / payload buffer size does not match the segments")
    dev, host, nseg = seg.args()
    _check(lib().tq_compress_segments_multi(_ptr_array(gs, "g"), len(gs), _dtype_code(gs[0]), d, dev, host, nseg,
                                            _ptr_array(params, "params"), bits, seed, first_worker, step,
                                            _ptr_array(payloads, "payload"), _stream()), "tq_compress_segments_multi")
    return payloads


def tq_decompress_aggregate_segments(payloads, params, seg, out, bits, weights=None, accumulate=False):
    d = out.numel()
    if out.dtype != torch.float32:
        raise TypeError("out must be float32")
    N = len(payloads)
    for p, q in zip(payloads, params):
        if p.numel() < payload_bytes(d, bits) or q.numel() != seg.nseg * PARAMS_BYTES:
            raise ValueError("payload / params buffer size does not match the segments")
    pp = (C.c_void_p * N)(*[_dev(p, "payload").value for p in payloads])
    qq = (C.c_void_p * N)(*[_dev(q, "params").value for q in params])
    ww = None if weights is None else (C.c_float * N)(*[float(w) for w in weights])
    dev, host, nseg = seg.args()
    _check(lib().tq_decompress_aggregate_segments(pp, qq, ww, N, d, dev, host, nseg, bits, int(bool(accumulate)),
                                                  _dev(out, "out"), _stream()), "tq_decompress_aggregate_segments")
    return out


def stats_to_numpy(stats):
    """Host copy of a stats buffer as a structured array (synchronises)."""
    return stats.cpu().numpy().view(STATS_DTYPE)


def params_to_numpy(params):
    """Host copy of a params buffer as a structured array (synchronises)."""
    return params.cpu().numpy().view(PARAMS_DTYPE)


def params_from_numpy(arr, device="cuda"):
    """Device buffer holding the given PARAMS_DTYPE-compatible records (same byte layout)."""
    raw = np.ascontiguousarray(arr).view(np.uint8).reshape(-1)
    return torch.from_numpy(raw.copy()).to(device)
