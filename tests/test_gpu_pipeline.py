"""The whole path on the GPU (stats -> params -> compress x N -> decode) against the oracle,
on scaled-down and on full-size benchmark workloads (synth.WORKLOADS)."""
import numpy as np
import pytest
import torch

from oracle import binding as O
from oracle import params as OP
from paper_2402_01798_amd import binding as B
from paper_2402_01798_amd import synth
from gpu_common import unpack_codes

pytestmark = pytest.mark.gpu


def run_device(wl, gs_dev, bits, grid, seed, step):
    d = gs_dev[0].numel()
    N = len(gs_dev)
    stats = [B.alloc_stats(d, wl.bucket_elems) for _ in range(N)]
    ws = B.alloc_stats_workspace(d, wl.bucket_elems)      # shared: the calls are ordered on one stream
    params = [B.alloc_params(d, wl.bucket_elems) for _ in range(N)]
    pays = [B.alloc_payload(d, bits) for _ in range(N)]
    out = torch.empty(d, dtype=torch.float32, device="cuda")
    for i in range(N):
        B.tq_stats(gs_dev[i], stats[i], ws, wl.bucket_elems, wl.g_min)
        B.tq_params(stats[i], params[i], bits, grid)
        B.tq_compress(gs_dev[i], params[i], pays[i], bits, seed, i, step, wl.bucket_elems, grid)
    B.tq_decompress_aggregate(pays, params, out, bits, wl.bucket_elems)
    torch.cuda.synchronize()
    return stats, params, pays, out


@pytest.mark.parametrize("name,d", [("cfg1", None), ("cfg2", 300_000), ("cfg3", (1 << 21) + 12_345),
                                    ("cfg4", (3 << 20) + 999), ("cfg5", 1_000_003)])
def test_whole_path_matches_oracle(name, d):
    wl = synth.WORKLOADS[name]
    d = wl.d if d is None else d
    N = min(wl.workers, 4)
    for bits in wl.bits:
        for grid in wl.grids:
            gs = [synth.make_gradient(wl, i, "cpu", d) for i in range(N)]
            gs_dev = [g.cuda() for g in gs]
            stats, params, pays, out = run_device(wl, gs_dev, bits, grid, seed=2024, step=5)
            P_dev, pay_or = [], []
            for i in range(N):
                g_np = synth.as_numpy(gs[i])
                S_or = O.stats(g_np, bucket_elems=wl.bucket_elems, g_min=wl.g_min)
                S_dev = B.stats_to_numpy(stats[i]).view(O.STATS_DTYPE)
                assert (S_dev["hist"] == S_or["hist"]).all() and (S_dev["absmax"] == S_or["absmax"]).all()
                assert (S_dev["n_tail"] == S_or["n_tail"]).all()
                P_or = OP.tq_params(S_or, bits, grid)
                Pd = B.params_to_numpy(params[i]).view(O.PARAMS_DTYPE)
                assert np.allclose(Pd["alpha"], P_or["alpha"], rtol=1e-6)
                assert np.allclose(Pd["level"], P_or["level"], rtol=1e-6, atol=0)
                assert (Pd["flags"] == P_or["flags"]).all()
                # codes: the oracle encodes with the very parameter bytes the device produced
                want = O.compress(g_np, Pd, 2024, i, 5, bucket_elems=wl.bucket_elems)
                assert (pays[i].cpu().numpy() == want).all()
                P_dev.append(Pd)
                pay_or.append(want)
            want_out = O.decompress_aggregate(pay_or, P_dev, d, bits, bucket_elems=wl.bucket_elems)
            got_out = out.cpu().numpy()
            scale = max(float(P["alpha"].max()) for P in P_dev)
            assert np.abs(got_out.astype(np.float64) - want_out).max() <= 1e-6 * scale
            assert (got_out == want_out).all()


@pytest.mark.parametrize("name,d,bits", [("cfg1", None, 3), ("cfg4", (2 << 20) + 777, 2), ("cfg2", 200_000, 4)])
def test_whole_path_with_the_biscaled_codebook(name, d, bits):
    """The BiScaled quantizer of the appendix through the whole path: parameters at 1e-6,
    then codes and averages bit for bit with the parameter bytes the device produced."""
    wl = synth.WORKLOADS[name]
    d = wl.d if d is None else d
    N = 3
    gs = [synth.make_gradient(wl, i, "cpu", d) for i in range(N)]
    stats, params, pays, out = run_device(wl, [g.cuda() for g in gs], bits, B.GRID_BISCALED, seed=99, step=4)
    P_dev, pay_or = [], []
    for i in range(N):
        g_np = synth.as_numpy(gs[i])
        S_or = O.stats(g_np, bucket_elems=wl.bucket_elems, g_min=wl.g_min)
        P_or = OP.tq_params(S_or, bits, B.GRID_BISCALED)
        Pd = B.params_to_numpy(params[i]).view(O.PARAMS_DTYPE)
        assert np.allclose(Pd["alpha"], P_or["alpha"], rtol=1e-6)
        assert np.allclose(Pd["level"], P_or["level"], rtol=1e-6, atol=0)
        assert (Pd["flags"] == P_or["flags"]).all() and (Pd["grid"] == B.GRID_BISCALED).all()
        want = O.compress(g_np, Pd, 99, i, 4, bucket_elems=wl.bucket_elems)
        assert (pays[i].cpu().numpy() == want).all()
        P_dev.append(Pd)
        pay_or.append(want)
    want_out = O.decompress_aggregate(pay_or, P_dev, d, bits, bucket_elems=wl.bucket_elems)
    assert (out.cpu().numpy() == want_out).all()


def test_cfg2_full_size_full_arrays():
    """Config 2 at its full size (11.2 M x 8 workers, uniform 2- and 4-bit) through the
    single-tensor entry points, one call per worker; every byte and every average is compared.
    (tests/test_gpu_full_size.py does the same through the batched entry points the benchmark
    times, for every configuration.)"""
    wl = synth.WORKLOADS["cfg2"]
    gs_dev = [synth.make_gradient(wl, i, "cuda") for i in range(wl.workers)]
    for bits in wl.bits:
        stats, params, pays, out = run_device(wl, gs_dev, bits, B.GRID_UNIFORM, seed=7, step=1)
        P_dev, pay_or = [], []
        for i in range(wl.workers):
            g_np = synth.as_numpy(gs_dev[i])
            S_dev = B.stats_to_numpy(stats[i]).view(O.STATS_DTYPE)
            assert S_dev.tobytes() == O.stats(g_np).tobytes()
            Pd = B.params_to_numpy(params[i]).view(O.PARAMS_DTYPE)
            want = O.compress(g_np, Pd, 7, i, 1)
            assert (pays[i].cpu().numpy() == want).all()
            P_dev.append(Pd)
            pay_or.append(want)
            print("cfg2 b=%d worker %d ok" % (bits, i), flush=True)
        want_out = O.decompress_aggregate(pay_or, P_dev, wl.d, bits)
        assert (out.cpu().numpy() == want_out).all()


@pytest.mark.parametrize("name", ["cfg3", "cfg4", "cfg5"])
def test_large_configs_sampled(name):
    """Configs 3-5 at full size: statistics compared in full where the oracle is
    quick, codes and averages on sampled elements computed by the oracle one at a time."""
    wl = synth.WORKLOADS[name]
    N = wl.workers if name != "cfg3" else 4            # 4 of the 16 workers keep the run short
    bits, grid = wl.bits[0], wl.grids[-1]
    gs_dev = [synth.make_gradient(wl, i, "cuda") for i in range(N)]
    print(name, "generated", flush=True)
    stats, params, pays, out = run_device(wl, gs_dev, bits, grid, seed=31337, step=2)
    rng = np.random.default_rng(5)
    d = wl.d
    idx = np.unique(np.concatenate([
        rng.integers(0, d, size=3000), np.arange(0, 64), np.arange(d - 64, d),
        (np.arange(1, 6) * (wl.bucket_elems or 2048))[:, None].repeat(2, 1).ravel() - np.array([1, 0] * 5)]))
    idx = idx[(idx >= 0) & (idx < d)]
    idx_dev = torch.from_numpy(idx).cuda()
    P_dev = [B.params_to_numpy(p).view(O.PARAMS_DTYPE) for p in params]
    levels = np.zeros((N, idx.size), dtype=np.float32)
    be = wl.bucket_elems
    for i in range(N):
        x = gs_dev[i][idx_dev].float().cpu().numpy()
        pay = pays[i].cpu().numpy()
        got = unpack_codes(pay, d, bits, idx)
        for t, e in enumerate(idx):
            P = P_dev[i][int(e) // be if be else 0: (int(e) // be if be else 0) + 1]
            want = O.quantize_one(float(x[t]), P, O.rand16(31337, i, 2, int(e)))
            assert got[t] == want, (name, i, int(e))
            levels[i, t] = P["level"][0][want]
        if i == 0:
            # statistics of worker 0, in full (one pass of the scalar oracle)
            S_or = O.stats(synth.as_numpy(gs_dev[0]), bucket_elems=be, g_min=wl.g_min)
            S_dev = B.stats_to_numpy(stats[0]).view(O.STATS_DTYPE)
            assert (S_dev["hist"] == S_or["hist"]).all() and (S_dev["n_tail"] == S_or["n_tail"]).all()
            assert (S_dev["absmax"] == S_or["absmax"]).all()
            assert np.allclose(S_dev["sum_log_tail"], S_or["sum_log_tail"], rtol=1e-6)
            P_or = OP.tq_params(S_or, bits, grid)
            assert np.allclose(P_dev[0]["alpha"], P_or["alpha"], rtol=1e-6)
            assert np.allclose(P_dev[0]["level"], P_or["level"], rtol=1e-6, atol=0)
        print(name, "worker", i, "ok", flush=True)
    acc = levels[0].copy()
    for i in range(1, N):
        acc = acc + levels[i]
    want_out = acc * np.float32(1.0 / N)
    got_out = out[idx_dev].cpu().numpy()
    assert (got_out == want_out).all()


def test_more_than_2_to_the_32_elements():
    """Element indices, byte offsets and tile counts beyond 32 bits: a bf16 tensor of
    2^32 + 6149 elements (five buckets of 2^30, the last one short and ragged), two workers.
    Codes and averages on sampled elements around every boundary, the short bucket's
    statistics in full, the others' by their totals."""
    wl = synth.WORKLOADS["cfg5"]
    d, be, bits, grid, N = (1 << 32) + 3 * 2048 + 5, 1 << 30, 2, B.GRID_NONUNIFORM, 2
    gs_dev = [synth.make_gradient(wl, i, "cuda", d) for i in range(N)]
    print("generated", flush=True)
    stats = [B.alloc_stats(d, be) for _ in range(N)]
    ws = B.alloc_stats_workspace(d, be)
    params = [B.alloc_params(d, be) for _ in range(N)]
    pays = [B.alloc_payload(d, bits) for _ in range(N)]
    out = torch.empty(d, dtype=torch.float32, device="cuda")
    for i in range(N):
        B.tq_stats(gs_dev[i], stats[i], ws, be, 1e-6)
        B.tq_params(stats[i], params[i], bits, grid)
        B.tq_compress(gs_dev[i], params[i], pays[i], bits, 4242, i, 7, be, grid)
    B.tq_decompress_aggregate(pays, params, out, bits, be)
    torch.cuda.synchronize()
    print("device path done", flush=True)
    S0 = B.stats_to_numpy(stats[0]).view(O.STATS_DTYPE)
    assert S0["n"].tolist() == [1 << 30] * 4 + [d - (4 << 30)]
    assert (S0["hist"].sum(axis=1) + S0["n_nonfinite"] == S0["n"]).all()
    tail = synth.as_numpy(gs_dev[0][4 << 30:])
    S_tail = O.stats(tail, g_min=1e-6)
    assert (S0["hist"][4] == S_tail["hist"][0]).all() and S0["absmax"][4] == S_tail["absmax"][0]
    assert S0["n_tail"][4] == S_tail["n_tail"][0]
    rng = np.random.default_rng(9)
    marks = np.array([1 << 30, 1 << 31, 3 << 30, 1 << 32, d], dtype=np.int64)
    idx = np.unique(np.concatenate([rng.integers(0, d, size=1500), np.arange(0, 16),
                                    (marks[:, None] + np.arange(-12, 12)[None, :]).ravel()]))
    idx = idx[(idx >= 0) & (idx < d)]
    idx_dev = torch.from_numpy(idx).cuda()
    levels = np.zeros((N, idx.size), dtype=np.float32)
    for i in range(N):
        P_all = B.params_to_numpy(params[i]).view(O.PARAMS_DTYPE)
        x = gs_dev[i][idx_dev].float().cpu().numpy()
        byte_lo = (idx * bits) >> 3
        pay_bytes = pays[i][torch.from_numpy(byte_lo).cuda()].cpu().numpy().astype(np.uint32)
        got = (pay_bytes >> ((idx * bits) & 7).astype(np.uint32)) & 3           # 2-bit codes never straddle a byte
        for t, e in enumerate(idx):
            P = P_all[int(e) // be: int(e) // be + 1]
            want = O.quantize_one(float(x[t]), P, O.rand16(4242, i, 7, int(e)))
            assert got[t] == want, (i, int(e))
            levels[i, t] = P["level"][0][want]
    want_out = (levels[0] + levels[1]) * np.float32(0.5)
    assert (out[idx_dev].cpu().numpy() == want_out).all()


def test_group_counter_beyond_32_bits():
    """Past 2^35 elements the group index that keys the random draws needs its high word, and
    with buckets of 2^30 + 128 elements a tile straddles that point, so some of its lanes are
    before the carry and some after.  Codes on sampled elements around it (compress only: a
    bf16 tensor of 2^35 + 10000 elements is 69 GB)."""
    wl = synth.WORKLOADS["cfg5"]
    d, be, bits = (1 << 35) + 10_000, (1 << 30) + 128, 2
    g = synth.make_gradient(wl, 0, "cuda", d)
    print("generated", flush=True)
    nb = B.num_buckets(d, be)
    from test_oracle_quantizer import make_params, NONUNIFORM_3
    P_all = np.concatenate([make_params(np.array(NONUNIFORM_3) * (1 + b % 3), O.GRID_NONUNIFORM) for b in range(nb)])
    pay = B.alloc_payload(d, bits)
    B.tq_compress(g, B.params_from_numpy(P_all), pay, bits, 0xFEEDFACE, 3, 11, be, B.GRID_NONUNIFORM)
    torch.cuda.synchronize()
    print("compressed", flush=True)
    rng = np.random.default_rng(3)
    marks = np.array([1 << 32, 1 << 35, 31 * be, 32 * be, d], dtype=np.int64)
    idx = np.unique(np.concatenate([rng.integers(0, d, size=1500), (1 << 35) + np.arange(-160, 2200, 7),
                                    (marks[:, None] + np.arange(-12, 12)[None, :]).ravel()]))
    idx = idx[(idx >= 0) & (idx < d)]
    x = g[torch.from_numpy(idx).cuda()].float().cpu().numpy()
    byte_lo = (idx * bits) >> 3
    pay_bytes = pay[torch.from_numpy(byte_lo).cuda()].cpu().numpy().astype(np.uint32)
    got = (pay_bytes >> ((idx * bits) & 7).astype(np.uint32)) & 3
    for t, e in enumerate(idx):
        P = P_all[int(e) // be: int(e) // be + 1]
        assert got[t] == O.quantize_one(float(x[t]), P, O.rand16(0xFEEDFACE, 3, 11, int(e))), int(e)
