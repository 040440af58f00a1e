"""Shared helpers of the GPU parity tests: same seeded inputs to the library and the oracle."""
import numpy as np
import torch

from oracle import binding as O
from oracle import params as OP
from paper_2402_01798_amd import binding as B
from paper_2402_01798_amd import synth


def small_gradient(wl_name, worker, d, dtype=None):
    """(device tensor, host numpy view) of the first d elements' recipe of a workload."""
    wl = synth.WORKLOADS[wl_name]
    g = synth.make_gradient(wl, worker, device="cpu", d=d, dtype=dtype)
    return g.cuda(), synth.as_numpy(g)


def oracle_params(g_np, bits, grid, bucket_elems=0, g_min=0.0, alpha_override=0.0):
    return OP.tq_params(O.stats(g_np, bucket_elems=bucket_elems, g_min=g_min), bits, grid, alpha_override)


def device_compress(g_dev, params_np, bits, seed, worker, step, bucket_elems=0, grid=None):
    """``grid`` = the family named to tq_compress (shapes the launch only); default: the records' own."""
    params_dev = B.params_from_numpy(params_np)
    payload = B.alloc_payload(g_dev.numel(), bits)
    payload.fill_(0xA5)                       # the library must overwrite every byte, padding included
    if grid is None:
        grid = int(np.asarray(params_np["grid"]).reshape(-1)[0])
    B.tq_compress(g_dev, params_dev, payload, bits, seed, worker, step, bucket_elems, grid)
    torch.cuda.synchronize()
    return payload


def unpack_codes(payload_np, d, bits, index=None):
    """Codes at the given element indices (all if None) from a little-endian b-bit stream."""
    if index is None:
        b = np.unpackbits(payload_np, bitorder="little")[: d * bits].reshape(d, bits)
        return (b.astype(np.uint32) << np.arange(bits, dtype=np.uint32)).sum(axis=1)
    index = np.asarray(index, dtype=np.int64)
    bitpos = index * bits
    word = np.zeros(index.size, dtype=np.uint32)
    for k in range(2):                        # a code spans at most two bytes
        word |= payload_np[np.minimum((bitpos >> 3) + k, payload_np.size - 1)].astype(np.uint32) << (8 * k)
    return (word >> (bitpos & 7).astype(np.uint32)) & ((1 << bits) - 1)
