"""tq_compress on the GPU against the oracle: packed bytes must be identical."""
import numpy as np
import pytest
import torch

from oracle import binding as O
from paper_2402_01798_amd import binding as B
from gpu_common import device_compress, oracle_params, small_gradient

pytestmark = pytest.mark.gpu

# sizes that span several 2048-element tiles and leave ragged tails of every kind
SIZES = [1, 5, 8, 9, 127, 128, 2047, 2048, 2049, 61_706, 3 * 2048 * 7 + 1234]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("grid", [B.GRID_UNIFORM, B.GRID_NONUNIFORM])
@pytest.mark.parametrize("d", SIZES)
def test_bytes_match_oracle_fp32(bits, grid, d):
    g_dev, g_np = small_gradient("cfg1", 1, d)
    P = oracle_params(g_np, bits, grid, g_min=1e-4 if d > 1000 else 0.0)
    got = device_compress(g_dev, P, bits, seed=0xC0FFEE1234, worker=1, step=3).cpu().numpy()
    want = O.compress(g_np, P, 0xC0FFEE1234, 1, 3)
    assert got.size == want.size
    assert (got == want).all()


@pytest.mark.parametrize("bits,grid", [(2, B.GRID_NONUNIFORM), (3, B.GRID_UNIFORM), (4, B.GRID_NONUNIFORM)])
@pytest.mark.parametrize("d", [9, 4100, 70_001])
def test_bytes_match_oracle_bf16(bits, grid, d):
    g_dev, g_np = small_gradient("cfg5", 0, d)
    assert g_dev.dtype == torch.bfloat16 and g_np.dtype == np.uint16
    P = oracle_params(g_np, bits, grid, g_min=1e-6)
    got = device_compress(g_dev, P, bits, 77, 0, 0).cpu().numpy()
    assert (got == O.compress(g_np, P, 77, 0, 0)).all()


@pytest.mark.parametrize("bits,grid", [(3, B.GRID_NONUNIFORM), (2, B.GRID_UNIFORM), (4, B.GRID_UNIFORM)])
@pytest.mark.parametrize("d,bucket", [(10_000, 2048), (10_000, 128), (3 * 4096, 4096), (70_000, 16_384), (5000, 8192)])
def test_buckets_match_oracle(bits, grid, d, bucket):
    g_dev, g_np = small_gradient("cfg4", 2, d)       # per-layer scales: buckets really differ
    P = oracle_params(g_np, bits, grid, bucket_elems=bucket)
    assert P.size == -(-d // bucket)
    got = device_compress(g_dev, P, bits, 5, 2, 9, bucket_elems=bucket).cpu().numpy()
    assert (got == O.compress(g_np, P, 5, 2, 9, bucket_elems=bucket)).all()


def test_special_values_and_seed_worker_step():
    d = 4096 + 37
    g_dev, g_np = small_gradient("cfg1", 0, d)
    g_np = g_np.copy()
    g_np[[0, 1, 2, 3, 4, 2050, d - 1]] = [np.nan, np.inf, -np.inf, 0.0, -0.0, np.nan, np.inf]
    g_np[10:20] = np.float32(1e-42)                   # denormals
    g_np[20:30] = [3e38, -3e38, 1e-30, -1e-30, 7.07e-4, -7.07e-4, 1e-4, -1e-4, 2.5e-4, 0.5]
    g_dev = torch.from_numpy(g_np).cuda()
    for bits, grid in [(3, B.GRID_UNIFORM), (3, B.GRID_NONUNIFORM), (2, B.GRID_NONUNIFORM), (4, B.GRID_UNIFORM)]:
        P = oracle_params(g_np, bits, grid, g_min=1e-4)
        seen = set()
        for seed, worker, step in [(0, 0, 0), (2 ** 64 - 1, 2 ** 32 - 1, 2 ** 32 - 1), (1, 0, 0), (0, 1, 0), (0, 0, 1)]:
            got = device_compress(g_dev, P, bits, seed, worker, step).cpu().numpy()
            assert (got == O.compress(g_np, P, seed, worker, step)).all()
            seen.add(got.tobytes())
        assert len(seen) == 5                        # every key component changes the stream


def test_hand_made_asymmetric_codebook():
    """The non-uniform path must follow any increasing table, not only mirrored ones."""
    d = 9000
    rng = np.random.default_rng(0)
    g_np = (rng.standard_normal(d) * 0.6).astype(np.float32)
    P = np.zeros(1, dtype=O.PARAMS_DTYPE)
    lv = np.array([-1.0, -0.9, -0.1, 0.0, 0.05, 0.3, 0.31, 1.0], dtype=np.float32)
    P["alpha"], P["bits"], P["s"], P["grid"] = 1.0, 3, 7, O.GRID_NONUNIFORM
    P["level"][0, :8] = lv
    P["inv_w"][0, :7] = (1.0 / np.diff(lv.astype(np.float64))).astype(np.float32)
    got = device_compress(torch.from_numpy(g_np).cuda(), P, 3, 9, 9, 9).cpu().numpy()
    assert (got == O.compress(g_np, P, 9, 9, 9)).all()
    # a cell of zero width (inv_w = 0) is skipped, never divided by
    lv2 = np.array([-1.0, -0.5, -0.5, 0.5], dtype=np.float32)
    P2 = np.zeros(1, dtype=O.PARAMS_DTYPE)
    P2["alpha"], P2["bits"], P2["s"], P2["grid"] = 1.0, 2, 3, O.GRID_NONUNIFORM
    P2["level"][0, :4] = lv2
    P2["inv_w"][0, :3] = [2.0, 0.0, 1.0]
    got = device_compress(torch.from_numpy(g_np).cuda(), P2, 2, 1, 1, 1).cpu().numpy()
    assert (got == O.compress(g_np, P2, 1, 1, 1)).all()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("lv", [[-1.0, -1.0, 1.0, 1.0],                          # empty first and last cell
                                [-1.0, -1.0, 0.0, 0.5, 0.5, 0.75, 1.0, 1.0],
                                [-1.0, -1.0, -1.0, 0.25, 0.25, 0.5, 0.5, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0]])
def test_empty_end_cells_and_values_beyond_the_threshold(lv, dtype):
    """Degenerate buckets give codebooks whose first or last cells are empty (levels repeated at -alpha
    or +alpha).  A value beyond -alpha is truncated ONTO the repeated level and so belongs to the cell
    above it (code 1 or 2, not 0): the truncation of Eq. (1) has to happen before the cell is looked
    up, also on the level-table path.  Values at, next to and far beyond +-alpha, infinities, NaN."""
    lv = np.array(lv, dtype=np.float32)
    s = lv.size - 1
    bits = {3: 2, 7: 3, 15: 4}[s]
    P = np.zeros(1, dtype=O.PARAMS_DTYPE)
    P["alpha"], P["bits"], P["s"], P["grid"] = 1.0, bits, s, O.GRID_NONUNIFORM
    P["level"][0, : s + 1] = lv
    width = np.diff(lv.astype(np.float64))
    P["inv_w"][0, :s] = np.where(width > 0, 1.0 / np.where(width > 0, width, 1.0), 0.0)
    d = 3 * 2048 + 77
    rng = np.random.default_rng(s)
    g = rng.standard_normal(d).astype(np.float32)
    special = np.array([1.0, -1.0, np.nextafter(np.float32(1), np.float32(2)), np.nextafter(np.float32(-1), np.float32(-2)),
                        1.5, -1.5, 3e38, -3e38, np.inf, -np.inf, np.nan, 0.0, -0.0, 0.25, 0.5, 0.75], dtype=np.float32)
    g[:: 97][: special.size] = special
    g[-16:] = special
    t = torch.from_numpy(g).to(dtype)
    g_np = t.view(torch.int16).numpy().view("uint16") if dtype == torch.bfloat16 else t.numpy()
    got = device_compress(t.cuda(), P, bits, 5, 1, 2).cpu().numpy()
    want = O.compress(g_np, P, 5, 1, 2)
    assert (got == want).all()
    codes = np.unpackbits(want, bitorder="little")[: d * bits].reshape(d, bits)
    codes = (codes.astype(np.uint32) << np.arange(bits, dtype=np.uint32)).sum(axis=1)
    below = np.nonzero(g < -1.0)[0]
    assert below.size > 0 and (codes[below] > 0).all()        # truncated onto the repeated level: the cell above


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("log2_width", [-20, -109, -110, -111, -112, -113, -120, 100, 120])
def test_very_narrow_and_very_wide_cells(log2_width, bits, dtype):
    """Cells so narrow that their reciprocal width is near the top of the binary32 range, and very wide
    ones: values spread over the codebook, at and next to every level, far beyond it, +-Inf, NaN; every
    code equal to the oracle's."""
    s = (1 << bits) - 1
    w = np.float64(2.0) ** log2_width
    lv = ((np.arange(s + 1) - s / 2.0) * w * (1.0 + 0.25 * (np.arange(s + 1) % 3))).astype(np.float32)   # unequal cells
    lv = np.sort(lv)
    P = np.zeros(1, dtype=O.PARAMS_DTYPE)
    P["alpha"], P["bits"], P["s"], P["grid"] = lv[-1], bits, s, O.GRID_NONUNIFORM
    P["level"][0, : s + 1] = lv
    width = np.diff(lv.astype(np.float64))
    with np.errstate(over="ignore"):
        iw = (1.0 / width).astype(np.float32)
    P["inv_w"][0, :s] = np.where(np.isfinite(iw), iw, 0.0)            # a reciprocal beyond the range is stored as 0
    d = 2 * 2048 + 333
    rng = np.random.default_rng(bits * 1000 + log2_width)
    g = (rng.uniform(-1.2, 1.2, d) * float(lv[-1])).astype(np.float32)
    near = np.concatenate([[l, np.nextafter(l, np.float32(np.inf)), np.nextafter(l, np.float32(-np.inf))] for l in lv])
    special = np.concatenate([near, np.array([0.0, -0.0, 3e38, -3e38, np.inf, -np.inf, np.nan], dtype=np.float32)])
    g[: special.size] = special
    g[-special.size:] = special
    t = torch.from_numpy(g.astype(np.float32)).to(dtype)
    g_np = t.view(torch.int16).numpy().view("uint16") if dtype == torch.bfloat16 else t.numpy()
    for seed in (1, 99):
        got = device_compress(t.cuda(), P, bits, seed, 3, 7).cpu().numpy()
        assert (got == O.compress(g_np, P, seed, 3, 7)).all()


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("d", [1, 5, 40, 41, 42, 43, 85, 86, 127, 128, 129, 2049, 4096 + 41])
def test_nothing_is_written_past_the_payload(bits, d):
    """The 3-byte groups of b = 3 can straddle the end of a short payload; the bytes behind
    the payload (here: a guard region of the same allocation) must stay untouched."""
    g_dev, g_np = small_gradient("cfg1", 0, d)
    P = oracle_params(g_np, bits, B.GRID_UNIFORM)
    nbytes = B.payload_bytes(d, bits)
    buf = torch.full((nbytes + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    B.tq_compress(g_dev, B.params_from_numpy(P), buf[:nbytes], bits, 77, 0, 0)
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    assert (got[nbytes:] == 0xA5).all()
    assert (got[:nbytes] == O.compress(g_np, P, 77, 0, 0)).all()


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("grid", [B.GRID_UNIFORM, B.GRID_NONUNIFORM])
def test_extreme_magnitudes_and_subnormal_reciprocals(bits, grid):
    """alpha = max|g| near the top of binary32 makes the reciprocal cell width subnormal (b < 4), and
    subnormal inputs sit next to it: both sides must keep subnormals (no flush to zero)."""
    d = 4099
    rng = np.random.default_rng(bits * 2 + grid)
    g_np = np.clip(rng.standard_normal(d) * 1e38, -3e38, 3e38).astype(np.float32)
    g_np[::7] = (rng.standard_normal(g_np[::7].size) * 1e-41).astype(np.float32)     # subnormal
    g_np[5] = np.float32(3.0e38)
    P = oracle_params(g_np, bits, grid, alpha_override=-1.0)
    assert float(P["inv_w"][0, 0]) < 3e-38           # subnormal at b = 2, 3; barely normal at b = 4
    got = device_compress(torch.from_numpy(g_np).cuda(), P, bits, seed=3, worker=0, step=0).cpu().numpy()
    assert (got == O.compress(g_np, P, 3, 0, 0)).all()
    # and the other end: everything subnormal, alpha at its floor
    tiny = (rng.standard_normal(d) * 1e-42).astype(np.float32)
    P = oracle_params(tiny, bits, grid)
    got = device_compress(torch.from_numpy(tiny).cuda(), P, bits, seed=3, worker=0, step=0).cpu().numpy()
    assert (got == O.compress(tiny, P, 3, 0, 0)).all()


def test_determinism_same_call_twice():
    g_dev, g_np = small_gradient("cfg2", 3, 200_000)
    P = oracle_params(g_np, 4, B.GRID_UNIFORM)
    a = device_compress(g_dev, P, 4, 11, 3, 1).cpu().numpy()
    b = device_compress(g_dev, P, 4, 11, 3, 1).cpu().numpy()
    assert (a == b).all()


@pytest.mark.parametrize("wl,dtype_name", [("cfg4", "fp32"), ("cfg5", "bf16")])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("family", [B.GRID_UNIFORM, B.GRID_NONUNIFORM])
def test_the_family_named_to_tq_compress_shapes_the_launch_only(wl, dtype_name, bits, family):
    """tq_compress's `grid` picks the number of tiles per workgroup; every bucket is encoded as its
    own record says.  So the payload must equal the oracle's whichever family is named, for
    records of either family -- over several workgroups of either shape, a short last bucket and
    a ragged end."""
    bucket = 3 * 4096 + 128
    d = 5 * bucket + 1234 + 5
    g_dev, g_np = small_gradient(wl, 1, d)
    P = oracle_params(g_np, bits, family, bucket_elems=bucket)
    want = O.compress(g_np, P, 21, 2, 9, bucket_elems=bucket)
    for named in (B.GRID_UNIFORM, B.GRID_NONUNIFORM, B.GRID_BISCALED):
        got = device_compress(g_dev, P, bits, 21, 2, 9, bucket, grid=named).cpu().numpy()
        assert (got == want).all(), (family, named)
