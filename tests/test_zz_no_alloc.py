"""tq_stats_static (the entry point that allocates nothing: its partial histograms go to a
scratch array the library holds on the device) against tq_stats, through the C ABI: the same
bytes, on two calls in a row, the second on a smaller input that leaves the first call's rows
behind in the scratch array."""
import numpy as np
import pytest
import torch

from paper_2402_01798_amd import binding as B
from gpu_common import small_gradient

pytestmark = pytest.mark.gpu


def both(g_dev, bucket, g_min):
    d = g_dev.numel()
    want = B.alloc_stats(d, bucket)
    ws = B.alloc_stats_workspace(d, bucket)
    B.tq_stats(g_dev, want, ws, bucket, g_min)
    got = B.alloc_stats(d, bucket)
    got.fill_(0x5A)                                     # must be overwritten in full
    B.tq_stats_static(g_dev, got, bucket, g_min)
    torch.cuda.synchronize()
    return got.cpu().numpy(), want.cpu().numpy()


@pytest.mark.parametrize("wl,first,second", [
    ("cfg4", ((3 << 20) + 999, 1 << 20, 0.0), (70_000, 16_384, 0.0)),       # several slices per bucket, then few
    ("cfg2", (2_000_003, 0, 0.0), (61_706, 0, 1e-4)),                       # one bucket cut into many slices
    ("cfg5", (5_000_000, 1 << 20, 1e-6), (1_000_003, 0, 1e-6)),             # bf16, tail terms
])
def test_static_scratch_gives_the_same_statistics_twice_in_a_row(wl, first, second):
    for d, bucket, g_min in (first, second):
        g_dev, _ = small_gradient(wl, 2, d)
        got, want = both(g_dev, bucket, g_min)
        assert got.tobytes() == want.tobytes(), (wl, d, bucket)
    # and once more on the first shape: the rows the smaller call left untouched are stale by now
    d, bucket, g_min = first
    g_dev, _ = small_gradient(wl, 3, d)
    got, want = both(g_dev, bucket, g_min)
    assert got.tobytes() == want.tobytes()


def test_sizes_beyond_the_scratch_array_are_refused():
    d, bucket = 128 * 4096, 128                         # 4096 buckets need more rows than the array holds
    assert B.stats_workspace_bytes(d, bucket) > (8 << 20)
    g = torch.zeros(d, dtype=torch.float32, device="cuda")
    st = B.alloc_stats(d, bucket)
    with pytest.raises(B.TqError) as e:
        B.tq_stats_static(g, st, bucket)
    assert e.value.code == B.EUNSUPPORTED
    # the largest benchmark shapes fit
    for dd, be in ((124_000_000, 1 << 20), (1_000_000_000, 0), (1_000_000_000, 1 << 20), (25_600_000, 1 << 20)):
        assert B.stats_workspace_bytes(dd, be) <= (8 << 20)
