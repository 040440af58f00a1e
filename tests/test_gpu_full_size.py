"""The benchmark configurations at FULL size, through the batched entry points bench.py times
(tq_stats_multi -> tq_params_multi -> tq_compress_multi -> tq_decompress_aggregate, all
workers of the configuration in one launch each), compared with the oracle on FULL arrays:
every statistics record, every payload byte, every averaged element.

The oracle is the scalar C code as it stands, run over disjoint element ranges on host
threads (16 by default: the box's share of cores for one GPU).  Parameters are compared at
1e-6 and the oracle then encodes with the very parameter bytes the device produced, so that a
last-bit difference in a level cannot flip a code.
"""
import os
import time

import numpy as np
import pytest
import torch

from oracle import binding as O
from oracle import params as OP
from paper_2402_01798_amd import binding as B
from paper_2402_01798_amd import synth

pytestmark = pytest.mark.gpu
THREADS = int(os.environ.get("TQ_ORACLE_THREADS", "16"))


def run_batched(wl, gs_dev, bits, grid, seed, step):
    """One step exactly as bench.py's Path.step launches it (mode 'batched')."""
    N, d, be = len(gs_dev), gs_dev[0].numel(), wl.bucket_elems
    stats = [B.alloc_stats(d, be) for _ in range(N)]
    ws = torch.empty(N * B.stats_workspace_bytes(d, be), dtype=torch.uint8, device="cuda")
    params = [B.alloc_params(d, be) for _ in range(N)]
    pays = [B.alloc_payload(d, bits) for _ in range(N)]
    for p in pays:
        p.fill_(0xA5)                                   # every byte must be overwritten
    out = torch.full((d,), float("nan"), dtype=torch.float32, device="cuda")
    B.tq_stats_multi(gs_dev, stats, ws, be, wl.g_min)
    B.tq_params_multi(stats, params, bits, grid)
    B.tq_compress_multi(gs_dev, params, pays, bits, seed, 0, step, be, grid)
    B.tq_decompress_aggregate(pays, params, out, bits, be)
    torch.cuda.synchronize()
    return stats, params, pays, out


def check_full(name, bits, grid, say, params_workers=2):
    wl = synth.WORKLOADS[name]
    N, d, be = wl.workers, wl.d, wl.bucket_elems
    seed, step = 0xC0FFEE + bits, 3
    t0 = time.time()
    gs_dev = [synth.make_gradient(wl, i, "cuda") for i in range(N)]
    stats, params, pays, out = run_batched(wl, gs_dev, bits, grid, seed, step)
    say("%s b=%d grid=%d: device path done at %.0f s" % (name, bits, grid, time.time() - t0))
    P_dev, pay_or = [], []
    for i in range(N):
        g_np = synth.as_numpy(gs_dev[i])
        gs_dev[i] = None                                 # free the device copy as we go
        S_or = O.stats(g_np, bucket_elems=be, g_min=wl.g_min, threads=THREADS)
        S_dev = B.stats_to_numpy(stats[i]).view(O.STATS_DTYPE)
        for f in ("hist", "n_nonfinite", "n", "n_tail", "absmax", "g_min"):
            assert (S_dev[f] == S_or[f]).all(), (name, i, f)
        assert np.allclose(S_dev["sum_log_tail"], S_or["sum_log_tail"], rtol=1e-6, atol=0)
        Pd = B.params_to_numpy(params[i]).view(O.PARAMS_DTYPE)
        if i < params_workers:
            P_or = OP.tq_params(S_dev, bits, grid)      # from the device's statistics bytes: the log-sum
                                                        # agrees to 1e-6 only, and alpha amplifies that
            assert np.allclose(Pd["alpha"], P_or["alpha"], rtol=1e-6)
            assert np.allclose(Pd["level"], P_or["level"], rtol=1e-6, atol=0)
            assert (Pd["flags"] == P_or["flags"]).all() and (Pd["grid"] == grid).all()
        want = O.compress(g_np, Pd, seed, i, step, bucket_elems=be, threads=THREADS)
        got = pays[i].cpu().numpy()
        assert got.size == want.size and (got == want).all(), (name, "payload of worker", i)
        P_dev.append(Pd)
        pay_or.append(want)
        del g_np, got
        say("  worker %d: statistics, parameters and %d payload bytes equal at %.0f s"
            % (i, want.size, time.time() - t0))
    want_out = O.decompress_aggregate(pay_or, P_dev, d, bits, bucket_elems=be, threads=THREADS)
    got_out = out.cpu().numpy()
    scale = max(float(P["alpha"].max()) for P in P_dev)
    for lo in range(0, d, 1 << 26):                      # in pieces: the fp64 difference of 10^9 values is 8 GB
        a, b = got_out[lo:lo + (1 << 26)], want_out[lo:lo + (1 << 26)]
        # the bar of the target: averages within 1e-6 (of the largest threshold: a purely relative
        # bound is ill-posed where +- levels cancel); what holds: the same adds in the same order
        assert np.abs(a.astype(np.float64) - b).max() <= 1e-6 * scale
        assert (a == b).all()
    say("  %d averages equal at %.0f s" % (d, time.time() - t0))


@pytest.fixture
def say(capsys):
    """Progress lines past pytest's capture: a long test must not look hung."""
    def _say(msg):
        with capsys.disabled():
            print(msg, flush=True)
    return _say


def test_cfg3_full_size_all_16_workers(say):
    """Config 3: 16 workers x 25.6 M fp32, non-uniform 3-bit, buckets of 2^20.  The compress launch
    is 1.6 GB (beyond the size up to which gradients are read with the non-temporal hint) and the
    decode runs 16 workers at b = 3 with a plainly stored 102 MB output."""
    check_full("cfg3", 3, B.GRID_NONUNIFORM, say, params_workers=16)


@pytest.mark.parametrize("grid", [B.GRID_UNIFORM, B.GRID_NONUNIFORM])
def test_cfg4_full_size_both_codebooks(grid, say):
    """Config 4: 8 workers x 124 M fp32, 2-bit, 119 buckets of 2^20 per worker (a 4 GB launch)."""
    check_full("cfg4", 2, grid, say)


@pytest.mark.parametrize("bits", [2, 4])
def test_cfg2_full_size_batched(bits, say):
    """Config 2: 8 workers x 11.2 M fp32, uniform 2- and 4-bit, one threshold per tensor."""
    check_full("cfg2", bits, B.GRID_UNIFORM, say, params_workers=8)


def test_cfg5_full_size(say):
    """Config 5: 4 workers x 10^9 bf16, non-uniform 2-bit, one codebook per tensor: 4 x 10^9
    element-encodes and 10^9 averages, all compared."""
    check_full("cfg5", 2, B.GRID_NONUNIFORM, say, params_workers=4)


def test_cfg4_full_size_one_record_per_layer(say):
    """Config 4 with one record per LAYER of its recipe (about 200 segments from 2^10 to 2^24 elements)
    through the batched segment calls bench.py times: 8 workers x 124 M fp32, uniform 2-bit.  The oracle's
    segment functions are scalar; the eight workers are checked on eight host threads."""
    from concurrent.futures import ThreadPoolExecutor
    wl = synth.WORKLOADS["cfg4"]
    N, d, bits, grid = wl.workers, wl.d, 2, B.GRID_UNIFORM
    seed, step = 0xC0FFEE, 5
    t0 = time.time()
    seg = B.Segments(synth.layer_segments(wl, d))
    gs_dev = [synth.make_gradient(wl, i, "cuda") for i in range(N)]
    stats = [torch.full((seg.nseg * B.STATS_BYTES,), 0x5A, dtype=torch.uint8, device="cuda") for _ in range(N)]
    ws = torch.empty(N * B.stats_segments_workspace_bytes(d, seg.nseg), dtype=torch.uint8, device="cuda")
    params = [torch.empty(seg.nseg * B.PARAMS_BYTES, dtype=torch.uint8, device="cuda") for _ in range(N)]
    pays = [B.alloc_payload(d, bits).fill_(0xA5) for _ in range(N)]
    out = torch.full((d,), float("nan"), dtype=torch.float32, device="cuda")
    B.tq_stats_segments_multi(gs_dev, seg, stats, ws, wl.g_min)
    B.tq_params_multi(stats, params, bits, grid)
    B.tq_compress_segments_multi(gs_dev, seg, params, pays, bits, seed, 0, step)
    B.tq_decompress_aggregate_segments(pays, params, seg, out, bits)
    torch.cuda.synchronize()
    say("cfg4 as %d layer segments: device path done at %.0f s" % (seg.nseg, time.time() - t0))
    gs_np = [synth.as_numpy(g) for g in gs_dev]
    del gs_dev

    def check_worker(i):
        S_or = O.stats_segments(gs_np[i], seg.host, g_min=wl.g_min)
        S_dev = B.stats_to_numpy(stats[i]).view(O.STATS_DTYPE)
        for f in ("hist", "n_nonfinite", "n", "n_tail", "absmax", "g_min"):
            assert (S_dev[f] == S_or[f]).all(), (i, f)
        assert np.allclose(S_dev["sum_log_tail"], S_or["sum_log_tail"], rtol=1e-6, atol=0)
        Pd = B.params_to_numpy(params[i]).view(O.PARAMS_DTYPE)
        P_or = OP.tq_params(S_dev, bits, grid)
        assert np.allclose(Pd["alpha"], P_or["alpha"], rtol=1e-6) and (Pd["flags"] == P_or["flags"]).all()
        want = O.compress_segments(gs_np[i], seg.host, Pd, seed, i, step)
        assert (pays[i].cpu().numpy() == want).all(), ("payload of worker", i)
        return Pd, want

    with ThreadPoolExecutor(max_workers=min(N, THREADS)) as ex:
        res = list(ex.map(check_worker, range(N)))
    say("  statistics, parameters and payloads of %d workers equal at %.0f s" % (N, time.time() - t0))
    want_out = O.decompress_aggregate_segments([r[1] for r in res], [r[0] for r in res], d, seg.host, bits)
    assert (out.cpu().numpy() == want_out).all()
    say("  %d averages equal at %.0f s" % (d, time.time() - t0))
