"""Batched entry points give exactly what the single-tensor calls give."""
import numpy as np
import pytest
import torch

from paper_2402_01798_amd import binding as B
from paper_2402_01798_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,d,count", [("cfg1", 61_706, 4), ("cfg2", 300_001, 8), ("cfg4", (2 << 20) + 777, 3),
                                          ("cfg5", 500_000, 5), ("cfg1", 9, 64)])
def test_multi_equals_single(name, d, count):
    wl = synth.WORKLOADS[name]
    be = wl.bucket_elems
    bits, grid = wl.bits[0], wl.grids[-1]
    gs = [synth.make_gradient(wl, i % 7, "cpu", d).cuda() for i in range(count)]
    # single-tensor path
    ws1 = B.alloc_stats_workspace(d, be)
    st1 = [B.alloc_stats(d, be) for _ in range(count)]
    pr1 = [B.alloc_params(d, be) for _ in range(count)]
    py1 = [B.alloc_payload(d, bits) for _ in range(count)]
    for i in range(count):
        B.tq_stats(gs[i], st1[i], ws1, be, wl.g_min)
        B.tq_params(st1[i], pr1[i], bits, grid)
        B.tq_compress(gs[i], pr1[i], py1[i], bits, 99, 10 + i, 3, be, grid)
    # batched path
    wsm = torch.empty(count * B.stats_workspace_bytes(d, be), dtype=torch.uint8, device="cuda")
    stm = [B.alloc_stats(d, be).fill_(0x11) for _ in range(count)]
    prm = [B.alloc_params(d, be).fill_(0x22) for _ in range(count)]
    pym = [B.alloc_payload(d, bits).fill_(0x33) for _ in range(count)]
    B.tq_stats_multi(gs, stm, wsm, be, wl.g_min)
    B.tq_params_multi(stm, prm, bits, grid)
    B.tq_compress_multi(gs, prm, pym, bits, 99, 10, 3, be, grid)
    torch.cuda.synchronize()
    for i in range(count):
        assert torch.equal(st1[i], stm[i]), ("stats", i)
        assert torch.equal(pr1[i], prm[i]), ("params", i)
        assert torch.equal(py1[i], pym[i]), ("payload", i)


def test_multi_rejects_bad_batches():
    d = 1000
    g = torch.zeros(d, device="cuda")
    st = B.alloc_stats(d)
    ws = B.alloc_stats_workspace(d)
    with pytest.raises(B.TqError) as e:
        B.tq_stats_multi([g, g], [st, st], ws)                 # workspace for one tensor only
    assert e.value.code == B.EINVAL
    with pytest.raises(B.TqError) as e:
        B.tq_params_multi([st] * 65, [B.alloc_params(d)] * 65, 2, 0)
    assert e.value.code == B.EUNSUPPORTED
