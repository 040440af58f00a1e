"""Variable-size segments on the GPU (one statistics record, threshold and codebook per layer,
Sec. V) against the oracle: statistics, parameters, payload bytes and averages."""
import numpy as np
import pytest
import torch

from oracle import binding as O
from oracle import params as OP
from paper_2402_01798_amd import binding as B
from paper_2402_01798_amd import synth
from gpu_common import small_gradient

pytestmark = pytest.mark.gpu


def run_segments(gs_dev, seg, bits, grid, g_min, seed, step):
    N, d = len(gs_dev), gs_dev[0].numel()
    stats = [torch.full((seg.nseg * B.STATS_BYTES,), 0x5A, dtype=torch.uint8, device="cuda") for _ in range(N)]
    ws = torch.full((B.stats_segments_workspace_bytes(d, seg.nseg),), 0xC3, dtype=torch.uint8, device="cuda")
    params = [torch.empty(seg.nseg * B.PARAMS_BYTES, dtype=torch.uint8, device="cuda") for _ in range(N)]
    pays = [B.alloc_payload(d, bits).fill_(0xA5) for _ in range(N)]
    out = torch.full((d,), float("nan"), dtype=torch.float32, device="cuda")
    for i in range(N):
        B.tq_stats_segments(gs_dev[i], seg, stats[i], ws, g_min)
        B.tq_params(stats[i], params[i], bits, grid)
        B.tq_compress_segments(gs_dev[i], seg, params[i], pays[i], bits, seed, i, step)
    B.tq_decompress_aggregate_segments(pays, params, seg, out, bits)
    torch.cuda.synchronize()
    return stats, params, pays, out


def run_segments_batched(gs_dev, seg, bits, grid, g_min, seed, step):
    """The same through the batched entry points: one launch per stage for all workers."""
    N, d = len(gs_dev), gs_dev[0].numel()
    stats = [torch.full((seg.nseg * B.STATS_BYTES,), 0x5A, dtype=torch.uint8, device="cuda") for _ in range(N)]
    ws = torch.full((N * B.stats_segments_workspace_bytes(d, seg.nseg),), 0xC3, dtype=torch.uint8, device="cuda")
    params = [torch.empty(seg.nseg * B.PARAMS_BYTES, dtype=torch.uint8, device="cuda") for _ in range(N)]
    pays = [B.alloc_payload(d, bits).fill_(0xA5) for _ in range(N)]
    out = torch.full((d,), float("nan"), dtype=torch.float32, device="cuda")
    B.tq_stats_segments_multi(gs_dev, seg, stats, ws, g_min)
    B.tq_params_multi(stats, params, bits, grid)
    B.tq_compress_segments_multi(gs_dev, seg, params, pays, bits, seed, 0, step)
    B.tq_decompress_aggregate_segments(pays, params, seg, out, bits)
    torch.cuda.synchronize()
    return stats, params, pays, out


def assert_same_bytes(a, b):
    for xs, ys in zip(a[:3], b[:3]):
        for x, y in zip(xs, ys):
            assert torch.equal(x, y)
    assert torch.equal(a[3], b[3])


def check_against_oracle(gs_np, seg, bits, grid, g_min, device, seed, step):
    stats, params, pays, out = device
    d = gs_np[0].size
    P_dev, pay_or = [], []
    for i, g_np in enumerate(gs_np):
        S_or = O.stats_segments(g_np, seg.host, g_min=g_min)
        S_dev = B.stats_to_numpy(stats[i]).view(O.STATS_DTYPE)
        for f in ("hist", "n_nonfinite", "n", "n_tail", "absmax", "g_min", "reserved"):
            assert (S_dev[f] == S_or[f]).all(), (i, f)
        assert np.allclose(S_dev["sum_log_tail"], S_or["sum_log_tail"], rtol=1e-6, atol=0)
        # parameters from the very statistics bytes the device produced: the log-sum is compared
        # at 1e-6 above, and the threshold amplifies such a difference several times
        P_or = OP.tq_params(S_dev, bits, grid)
        Pd = B.params_to_numpy(params[i]).view(O.PARAMS_DTYPE)
        assert np.allclose(Pd["alpha"], P_or["alpha"], rtol=1e-6)
        assert np.allclose(Pd["level"], P_or["level"], rtol=1e-6, atol=0)
        assert (Pd["flags"] == P_or["flags"]).all()
        want = O.compress_segments(g_np, seg.host, Pd, seed, i, step)
        assert (pays[i].cpu().numpy() == want).all(), ("payload", i)
        P_dev.append(Pd)
        pay_or.append(want)
    want_out = O.decompress_aggregate_segments(pay_or, P_dev, d, seg.host, bits)
    assert (out.cpu().numpy() == want_out).all()


@pytest.mark.parametrize("wl,g_min", [("cfg4", 0.0), ("cfg5", 1e-6), ("cfg1", 1e-4)])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("grid", [B.GRID_UNIFORM, B.GRID_NONUNIFORM])
def test_ragged_segments_match_oracle(wl, g_min, bits, grid):
    """Segments from 128 elements (many inside one tile) to several tiles and chunks, the last one
    ragged (41 elements past a multiple of 128: a 3-bit payload then ends inside a group)."""
    offs = [0, 128, 256, 1152, 2048, 2176, 6144, 6272, 140_032, 140_160, 300_032, 300_032 + 41]
    seg = B.Segments(offs)
    N = 3
    gs = [small_gradient(wl, i, seg.d) for i in range(N)]
    device = run_segments([g[0] for g in gs], seg, bits, grid, g_min, seed=77, step=2)
    check_against_oracle([g[1] for g in gs], seg, bits, grid, g_min, device, 77, 2)
    # one launch per stage for the three workers: the same bytes
    assert_same_bytes(device, run_segments_batched([g[0] for g in gs], seg, bits, grid, g_min, seed=77, step=2))


def test_layers_of_config_4_as_segments():
    """The layer recipe of config 4 (layers of 2^U[10,24] elements, each with its own scale) with one
    record per LAYER instead of per 2^20-element bucket: the first 30 M elements, 2 workers, 2-bit
    non-uniform."""
    wl = synth.WORKLOADS["cfg4"]
    d = 30_000_000
    seg = B.Segments(synth.layer_segments(wl, d))
    assert seg.nseg > 5 and seg.d == d
    gs_dev = [synth.make_gradient(wl, i, "cuda", d) for i in range(2)]
    device = run_segments(gs_dev, seg, 2, B.GRID_NONUNIFORM, 0.0, seed=5, step=1)
    check_against_oracle([synth.as_numpy(g) for g in gs_dev], seg, 2, B.GRID_NONUNIFORM, 0.0, device, 5, 1)
    # every layer got a threshold of its own scale: they spread over orders of magnitude
    alphas = B.params_to_numpy(device[1][0])["alpha"]
    assert alphas.max() / alphas.min() > 100


def test_equal_segments_give_what_the_bucketed_calls_give():
    d, be, bits = 5 * 4096 + 1000, 4096, 3
    g_dev, _ = small_gradient("cfg3", 0, d)
    seg = B.Segments(list(range(0, d, be)) + [d])
    stats, params, pays, out = run_segments([g_dev], seg, bits, B.GRID_NONUNIFORM, 1e-5, seed=9, step=9)
    st = B.alloc_stats(d, be)
    B.tq_stats(g_dev, st, B.alloc_stats_workspace(d, be), be, 1e-5)
    pr = B.alloc_params(d, be)
    B.tq_params(st, pr, bits, B.GRID_NONUNIFORM)
    py = B.alloc_payload(d, bits)
    B.tq_compress(g_dev, pr, py, bits, 9, 0, 9, be, B.GRID_NONUNIFORM)
    o2 = torch.empty(d, dtype=torch.float32, device="cuda")
    B.tq_decompress_aggregate([py], [pr], o2, bits, be)
    torch.cuda.synchronize()
    assert torch.equal(st, stats[0]) and torch.equal(pr, params[0]) and torch.equal(py, pays[0]) and torch.equal(o2, out)


def test_weights_and_accumulate():
    offs = [0, 256, 4096 + 128, 9000]
    seg = B.Segments(offs)
    N, bits = 2, 4
    gs = [small_gradient("cfg2", i, seg.d) for i in range(N)]
    stats, params, pays, out = run_segments([g[0] for g in gs], seg, bits, B.GRID_UNIFORM, 0.0, seed=3, step=0)
    w = [0.75, 0.25]
    acc = torch.full((seg.d,), 2.0, dtype=torch.float32, device="cuda")
    B.tq_decompress_aggregate_segments(pays, params, seg, acc, bits, weights=w, accumulate=True)
    torch.cuda.synchronize()
    P = [B.params_to_numpy(p).view(O.PARAMS_DTYPE) for p in params]
    want = O.decompress_aggregate_segments([p.cpu().numpy() for p in pays], P, seg.d, seg.host, bits, weights=w,
                                           out=np.full(seg.d, 2.0, dtype=np.float32))
    assert (acc.cpu().numpy() == want).all()


def test_a_malformed_host_table_is_refused():
    g = torch.zeros(1000, device="cuda")
    for offs in ([0, 100, 1000], [0, 512, 384, 1000], [128, 1000], [0, 512, 512, 1000], [0, 512, 900]):
        seg = B.Segments(offs)
        st = torch.empty(seg.nseg * B.STATS_BYTES, dtype=torch.uint8, device="cuda")
        ws = torch.empty(max(1, B.stats_segments_workspace_bytes(1000, seg.nseg)), dtype=torch.uint8, device="cuda")
        with pytest.raises(B.TqError) as e:
            B.tq_stats_segments(g, seg, st, ws)
        assert e.value.code == B.EINVAL


def test_more_workers_than_the_fast_decode_takes():
    """17 workers: the aggregate goes through the general segment kernel (plain level rows for up to
    64 workers) instead of the two-tiles-per-workgroup one."""
    offs = [0, 384, 2048, 2048 + 4096 * 3, 19_968, 19_968 + 128 * 9, 33_001]
    seg = B.Segments(offs)
    N, bits = 17, 3
    gs = [small_gradient("cfg3", i, seg.d) for i in range(N)]
    device = run_segments_batched([g[0] for g in gs], seg, bits, B.GRID_NONUNIFORM, 1e-5, seed=11, step=4)
    check_against_oracle([g[1] for g in gs], seg, bits, B.GRID_NONUNIFORM, 1e-5, device, 11, 4)
