"""tq_stats and tq_params on the GPU against the oracle."""
import numpy as np
import pytest
import torch

from oracle import binding as O
from oracle import params as OP
from paper_2402_01798_amd import binding as B
from gpu_common import small_gradient

pytestmark = pytest.mark.gpu


def device_stats(g_dev, bucket=0, g_min=0.0):
    st = B.alloc_stats(g_dev.numel(), bucket)
    st.fill_(0x5A)                                   # must be overwritten in full
    ws = B.alloc_stats_workspace(g_dev.numel(), bucket)
    ws.fill_(0xC3)                                   # need not be cleared by the caller
    B.tq_stats(g_dev, st, ws, bucket, g_min)
    torch.cuda.synchronize()
    return st


def assert_stats_equal(got, want):
    for f in ("hist", "n_nonfinite", "n", "n_tail", "reserved"):
        assert (got[f] == want[f]).all(), f
    assert (got["absmax"] == want["absmax"]).all()
    assert (got["g_min"] == want["g_min"]).all()
    assert np.allclose(got["sum_log_tail"], want["sum_log_tail"], rtol=1e-6, atol=0)


@pytest.mark.parametrize("wl,dtype", [("cfg1", None), ("cfg2", None), ("cfg5", None)])
@pytest.mark.parametrize("d,bucket", [(1, 0), (7, 0), (2049, 0), (61_706, 0), (200_001, 0), (70_000, 16_384), (10_000, 128), (40_000, 32_768)])
@pytest.mark.parametrize("g_min", [0.0, 1e-4])
def test_stats_match_oracle(wl, dtype, d, bucket, g_min):
    g_dev, g_np = small_gradient(wl, 1, d)
    got = B.stats_to_numpy(device_stats(g_dev, bucket, g_min))
    want = O.stats(g_np, bucket_elems=bucket, g_min=g_min)
    assert_stats_equal(got, want)


def test_stats_special_values():
    d = 20_000
    g_dev, g_np = small_gradient("cfg1", 0, d)
    g_np = g_np.copy()
    g_np[[0, 5, 4097, d - 1]] = [np.nan, np.inf, -np.inf, np.nan]
    g_np[100:110] = 0.0
    g_np[110:120] = np.float32(1e-42)
    g_np[120:124] = [3e38, 70000.0, 65536.0, 2.0 ** -40]
    got = B.stats_to_numpy(device_stats(torch.from_numpy(g_np).cuda(), 0, 1e-4))
    assert_stats_equal(got, O.stats(g_np, g_min=1e-4))
    zeros = torch.zeros(5000, device="cuda")
    got = B.stats_to_numpy(device_stats(zeros))
    assert got["hist"][0, 0] == 5000 and got["absmax"][0] == 0.0


PARAM_CASES = [("cfg1", 1e-4), ("cfg1", 0.0), ("cfg2", 0.0), ("cfg3", 1e-5), ("cfg4", 0.0), ("cfg5", 1e-6)]


def assert_params_close(got, want):
    for f in ("bits", "s", "grid", "flags"):
        assert (got[f] == want[f]).all(), (f, got[f], want[f])
    for f in ("alpha", "gamma_hat", "rho_hat", "g_min"):
        assert np.allclose(got[f], want[f], rtol=1e-6, atol=0), (f, got[f], want[f])
    assert np.allclose(got["level"], want["level"], rtol=1e-6, atol=0)
    assert np.allclose(got["inv_w"], want["inv_w"], rtol=2e-6, atol=0)


@pytest.mark.parametrize("wl,g_min", PARAM_CASES)
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("grid", [B.GRID_UNIFORM, B.GRID_NONUNIFORM, B.GRID_BISCALED])
def test_params_match_oracle(wl, g_min, bits, grid):
    d, bucket = 300_000, 65_536
    g_dev, g_np = small_gradient(wl, 0, d)
    st = device_stats(g_dev, bucket, g_min)
    pr = B.alloc_params(d, bucket)
    pr.fill_(0x77)
    B.tq_params(st, pr, bits, grid)
    torch.cuda.synchronize()
    got = B.params_to_numpy(pr)
    want = OP.tq_params(B.stats_to_numpy(st).view(O.STATS_DTYPE), bits, grid)
    assert_params_close(got, want)


@pytest.mark.parametrize("override", [-1.0, 3.3e-4])
def test_params_override_and_degenerate(override):
    d = 50_000
    g_dev, g_np = small_gradient("cfg1", 0, d)
    st = device_stats(g_dev, 0, 1e-4)
    for grid in (B.GRID_UNIFORM, B.GRID_NONUNIFORM, B.GRID_BISCALED):
        pr = B.alloc_params(d)
        B.tq_params(st, pr, 3, grid, override)
        torch.cuda.synchronize()
        want = OP.tq_params(B.stats_to_numpy(st).view(O.STATS_DTYPE), 3, grid, override)
        assert_params_close(B.params_to_numpy(pr), want)
    for data in (torch.zeros(4096, device="cuda"), torch.full((4096,), 0.25, device="cuda"),
                 torch.full((4096,), float("nan"), device="cuda")):
        st = device_stats(data)
        for grid in (B.GRID_UNIFORM, B.GRID_NONUNIFORM, B.GRID_BISCALED):
            pr = B.alloc_params(4096)
            B.tq_params(st, pr, 2, grid)
            torch.cuda.synchronize()
            want = OP.tq_params(B.stats_to_numpy(st).view(O.STATS_DTYPE), 2, grid)
            assert_params_close(B.params_to_numpy(pr), want)
            # a threshold the caller gives is used even when there is nothing to design from
            B.tq_params(st, pr, 2, grid, 0.5)
            torch.cuda.synchronize()
            want = OP.tq_params(B.stats_to_numpy(st).view(O.STATS_DTYPE), 2, grid, 0.5)
            got = B.params_to_numpy(pr)
            assert float(got["alpha"][0]) == 0.5
            assert_params_close(got, want)


def test_cfg1_alpha_is_the_closed_form_value():
    """Config 1 (gamma = 3, x_min = 1e-4, s = 7): alpha* = 1e-4 sqrt(50) on the device too."""
    wl_d = 61_706
    g_dev, _ = small_gradient("cfg1", 0, wl_d)
    st = device_stats(g_dev, 0, 1e-4)
    pr = B.alloc_params(wl_d)
    B.tq_params(st, pr, 3, B.GRID_UNIFORM)
    torch.cuda.synchronize()
    P = B.params_to_numpy(pr)
    assert float(P["alpha"][0]) == pytest.approx(7.0710678e-4, rel=0.03)   # sampling error of gamma-hat
    assert float(P["gamma_hat"][0]) == pytest.approx(3.0, abs=0.05)
    assert float(P["rho_hat"][0]) == pytest.approx(0.5, abs=1e-3)


@pytest.mark.parametrize("wl,d,bucket,count,g_min", [
    ("cfg4", 1_000_003, 32_768 + 128 * 3, 3, 0.0),      # buckets that are no multiple of a 4096-element tile
    ("cfg3", 1_000_003, 32_768 + 128 * 3, 2, 1e-5),     # the same with tail terms
    ("cfg5", 2_500_001, 1 << 20, 4, 1e-6),              # bf16, 1024 shares over 4 tensors, a ragged end
    ("cfg4", 9_000_000, 32_768, 2, 0.0),                # more buckets (550) than shares: rows added per boundary
    ("cfg2", 3_000_000, 0, 1, 0.0),                     # one bucket over 183 shares: the wide second kernel
    ("cfg1", 70_000, 65_536, 5, 1e-4),                  # shares that span tensors of the batch
])
def test_large_buckets_cut_into_equal_shares(wl, d, bucket, count, g_min):
    """Buckets of 32768 elements or more: the batch is cut into equal shares of tiles whatever the buckets
    are; records inside one share are written directly, the others added from partial rows."""
    gs = [small_gradient(wl, 10 + i, d) for i in range(count)]
    stats = [B.alloc_stats(d, bucket).fill_(0x5A) for _ in range(count)]
    ws = torch.full((count * B.stats_workspace_bytes(d, bucket),), 0xC3, dtype=torch.uint8, device="cuda")
    B.tq_stats_multi([g[0] for g in gs], stats, ws, bucket, g_min)
    torch.cuda.synchronize()
    for i in range(count):
        assert_stats_equal(B.stats_to_numpy(stats[i]), O.stats(gs[i][1], bucket_elems=bucket, g_min=g_min))
        # one tensor alone gives the same bytes (another partition of the same work)
        single = device_stats(gs[i][0], bucket, g_min)
        assert torch.equal(single, stats[i])


@pytest.mark.parametrize("g_min", [2.0 ** -40, 2.0 ** -40 * (1 + 2.0 ** -20), 0.5, 0.53125, 0.531250059604645,
                                   61439.99609375, 61440.0, 65536.0, 65535.99609375, 1.0e5, 3.0e38])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_tail_terms_for_thresholds_on_and_between_bin_edges(dtype, g_min):
    """The tail's exponent sum is taken from the histogram (a bin lies inside one octave) and the tail
    count of g_min's own bin; the last bin (65536 and up) spans octaves and is taken element by element.
    Thresholds on bin edges, next to them, inside the last bin and above everything; values spread over
    every octave from 2^-45 to 2^100."""
    d = 70_000
    g_dev, g_np = small_gradient("cfg1", 5, d)
    g_np = g_np.astype(np.float32).copy()
    rng = np.random.default_rng(17)
    idx = rng.choice(d, 6000, replace=False)
    mags = np.exp2(rng.uniform(-45, 100, idx.size)).astype(np.float32)
    g_np[idx] = mags * rng.choice([-1.0, 1.0], idx.size).astype(np.float32)
    g_np[idx[:12]] = [61440.0, -61440.0, 61439.99609375, 65536.0, 65535.99609375, 0.5, 0.53125, -0.5, 2.0 ** -40,
                      np.inf, np.nan, 3.0e38]
    if dtype == "bf16":                                  # the oracle reads the bit patterns the device sees
        g_t = torch.from_numpy(g_np).to(torch.bfloat16)
        g_np = g_t.view(torch.int16).numpy().view(np.uint16)
    else:
        g_t = torch.from_numpy(g_np)
    def equal(got, want):
        # the counts exactly; the log-sum to 1e-6, plus what one group's logarithm can be off by when the
        # tail is a handful of elements next to the threshold and the sum itself is next to zero
        for f in ("hist", "n_nonfinite", "n", "n_tail", "absmax", "g_min"):
            assert (got[f] == want[f]).all(), f
        assert np.allclose(got["sum_log_tail"], want["sum_log_tail"], rtol=1e-6, atol=4e-7)

    equal(B.stats_to_numpy(device_stats(g_t.cuda(), 0, g_min)), O.stats(g_np, g_min=g_min))
    # small buckets: the other kernel
    equal(B.stats_to_numpy(device_stats(g_t.cuda(), 16_384, g_min)), O.stats(g_np, bucket_elems=16_384, g_min=g_min))
