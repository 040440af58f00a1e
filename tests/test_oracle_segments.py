"""Variable-size segments in the oracle (Sec. V: layers are quantized independently): pinned to
the bucketed functions, which are pinned elsewhere -- equal-sized segments ARE buckets, and a
segment on its own is a tensor of its own apart from where its random draws and payload bits
sit in the flat gradient."""
import numpy as np
import pytest

from oracle import binding as O
from oracle import params as OP


def gradient(d, seed):
    rng = np.random.default_rng(seed)
    return (1e-3 * rng.uniform(size=d) ** -0.6 * rng.choice([-1.0, 1.0], size=d)).astype(np.float32)


@pytest.mark.parametrize("bits,grid", [(2, O.GRID_UNIFORM), (3, O.GRID_NONUNIFORM), (4, O.GRID_UNIFORM)])
def test_equal_segments_are_buckets(bits, grid):
    d, be = 5 * 1024 + 300, 1024
    g = gradient(d, 1)
    off = np.array(list(range(0, d, be)) + [d], dtype=np.uint64)
    S_b = O.stats(g, bucket_elems=be, g_min=1e-3)
    S_s = O.stats_segments(g, off, g_min=1e-3)
    assert S_b.tobytes() == S_s.tobytes()
    P = OP.tq_params(S_s, bits, grid)
    pay_b = O.compress(g, P, 5, 2, 7, bucket_elems=be)
    pay_s = O.compress_segments(g, off, P, 5, 2, 7)
    assert (pay_b == pay_s).all()
    out_b = O.decompress_aggregate([pay_b, pay_b], [P, P], d, bits, bucket_elems=be)
    out_s = O.decompress_aggregate_segments([pay_s, pay_s], [P, P], d, off, bits)
    assert (out_b == out_s).all()


def test_ragged_segments_element_by_element():
    """Each element is encoded with ITS segment's record and ITS index in the flat gradient."""
    d = 128 * 37 + 5
    off = np.array([0, 128, 128 * 3, 128 * 20, 128 * 21, d], dtype=np.uint64)
    g = gradient(d, 2)
    S = O.stats_segments(g, off)
    for s in range(off.size - 1):
        lo, hi = int(off[s]), int(off[s + 1])
        assert S[s].tobytes() == O.stats(g[lo:hi])[0].tobytes()
    P = OP.tq_params(S, 3, O.GRID_NONUNIFORM)
    assert len({float(a) for a in P["alpha"]}) == off.size - 1        # every segment its own threshold
    pay = O.compress_segments(g, off, P, 11, 3, 4)
    codes = np.unpackbits(pay, bitorder="little")[: d * 3].reshape(d, 3)
    codes = (codes.astype(np.uint32) << np.arange(3, dtype=np.uint32)).sum(axis=1)
    rng = np.random.default_rng(0)
    probe = np.unique(np.concatenate([rng.integers(0, d, 300), off[:-1].astype(np.int64), off[1:].astype(np.int64) - 1]))
    for e in probe:
        s = int(np.searchsorted(off, e, side="right")) - 1
        assert codes[e] == O.quantize_one(float(g[e]), P[s:s + 1], O.rand16(11, 3, 4, int(e)))
    out = O.decompress_aggregate_segments([pay], [P], d, off, 3)
    for e in probe:
        s = int(np.searchsorted(off, e, side="right")) - 1
        assert out[e] == P["level"][s][codes[e]]


def test_bad_segment_tables_are_rejected():
    g = gradient(1000, 3)
    for off in ([0, 100, 1000],            # an interior offset that is not a multiple of 128
                [0, 512, 384, 1000],       # not ascending
                [128, 1000],               # does not start at 0
                [0, 512, 512, 1000]):      # an empty segment
        with pytest.raises(ValueError):
            O.stats_segments(g, np.array(off, dtype=np.uint64))
