"""Pins for the wire format ("encode it using b bits", Sec. III-A) and the server
step of Alg. 1 (g_bar = sum_i w_i g_hat_i)."""
import numpy as np
import pytest

from oracle import binding as O
from test_oracle_quantizer import NONUNIFORM_7, make_params, uniform_params


def unpack_le(payload, d, bits):
    """Independent reader: numpy's little-endian bit unpacking."""
    b = np.unpackbits(np.asarray(payload, dtype=np.uint8), bitorder="little")
    b = b[: d * bits].reshape(d, bits).astype(np.uint32)
    return (b << np.arange(bits, dtype=np.uint32)).sum(axis=1)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("d", [1, 7, 8, 9, 127, 128, 1000, 4099])
def test_stream_layout_size_padding_and_round_trip(bits, d):
    rng = np.random.default_rng(d * 10 + bits)
    g = rng.standard_normal(d).astype(np.float32)
    P = uniform_params(1.5, bits)
    payload = O.compress(g, P, seed=5, worker=2, step=9)
    nbytes = (d * bits + 7) // 8
    assert payload.size == (nbytes + 15) // 16 * 16 == O.payload_bytes(d, bits)
    allbits = np.unpackbits(payload, bitorder="little")
    assert not allbits[d * bits:].any()                      # pad bits are zero
    codes = unpack_le(payload, d, bits)
    want = np.array([O.quantize_one(float(g[e]), P, O.rand16(5, 2, 9, e)) for e in range(d)])
    assert (codes == want).all()
    # dequantize reads the same stream back
    q = O.dequantize(payload, P, d, bits)
    assert (q == P["level"][0][codes]).all()


def test_draw_depends_on_the_global_index_not_on_the_bucket():
    d, B = 1024, 256
    rng = np.random.default_rng(0)
    g = rng.standard_normal(d).astype(np.float32)
    P1 = uniform_params(1.0, 3)
    P4 = np.concatenate([P1] * 4)
    a = O.compress(g, P1, 11, 0, 0)
    b = O.compress(g, P4, 11, 0, 0, bucket_elems=B)
    assert (a == b).all()
    # different parameters per bucket are honoured bucket by bucket
    P4b = np.concatenate([uniform_params(a_, 3) for a_ in (0.5, 1.0, 2.0, 4.0)])
    c = unpack_le(O.compress(g, P4b, 11, 0, 0, bucket_elems=B), d, 3)
    for j, a_ in enumerate((0.5, 1.0, 2.0, 4.0)):
        seg = slice(j * B, (j + 1) * B)
        want = unpack_le(O.compress(np.concatenate([np.zeros(j * B, np.float32), g[seg]]),
                                    uniform_params(a_, 3), 11, 0, 0), (j + 1) * B, 3)[seg]
        assert (c[seg] == want).all()


def test_invalid_layouts_are_rejected():
    g = np.zeros(300, dtype=np.float32)
    with pytest.raises(ValueError):
        O.compress(g, np.concatenate([uniform_params(1.0, 2)] * 3), 0, 0, 0, bucket_elems=100)
    with pytest.raises(ValueError):
        O.stats(g, bucket_elems=100)


def test_aggregate_of_identical_streams_returns_the_levels():
    """sum_i (1/N) L[c] = L[c]; exact in binary32 for dyadic levels and N a power of two."""
    d = 777
    rng = np.random.default_rng(1)
    g = (rng.standard_normal(d) * 0.4).astype(np.float32)
    P = make_params([-1, -0.5, -0.25, -0.0625, 0.0625, 0.25, 0.5, 1], O.GRID_NONUNIFORM)
    pay = O.compress(g, P, 3, 0, 0)
    for N in (1, 2, 8):
        out = O.decompress_aggregate([pay] * N, [P] * N, d, 3)
        assert (out == O.dequantize(pay, P, d, 3)).all()


def test_aggregate_is_the_weighted_sum_of_alg1():
    d = 1500
    rng = np.random.default_rng(2)
    N = 5
    gs = [(rng.standard_normal(d) * (0.1 + i)).astype(np.float32) for i in range(N)]
    Ps = [uniform_params(0.3 + 0.5 * i, 4) for i in range(N)]
    pays = [O.compress(gs[i], Ps[i], 8, i, 4) for i in range(N)]
    deq = np.stack([O.dequantize(pays[i], Ps[i], d, 4).astype(np.float64) for i in range(N)])
    out = O.decompress_aggregate(pays, Ps, d, 4)
    assert np.allclose(out, deq.mean(axis=0), rtol=0, atol=4 * 2.0 ** -24 * np.abs(deq).sum(axis=0).max())
    w = np.array([0.1, 0.2, 0.3, 0.25, 0.15], dtype=np.float32)
    outw = O.decompress_aggregate(pays, Ps, d, 4, weights=w)
    assert np.allclose(outw, (w[:, None].astype(np.float64) * deq).sum(axis=0), rtol=0,
                       atol=4 * 2.0 ** -24 * np.abs(deq).sum(axis=0).max())
    # accumulate mode adds to what is there
    base = rng.standard_normal(d).astype(np.float32)
    acc = O.decompress_aggregate(pays, Ps, d, 4, out=base.copy())
    assert (acc == base + out).all()


def test_lossless_when_the_input_lies_on_the_codebook_and_is_not_truncated():
    """Eq. (2) with p_r in {0,1}: compress then aggregate over one worker is the identity."""
    P = uniform_params(3.5, 3)                      # levels -3.5, -2.5, ..., 3.5 exactly
    rng = np.random.default_rng(4)
    g = P["level"][0, rng.integers(0, 8, size=999)].copy()
    out = O.decompress_aggregate([O.compress(g, P, 1, 0, 0)], [P], g.size, 3)
    assert (out == g).all()


def test_aggregated_average_is_unbiased_and_its_error_shrinks_like_one_over_n():
    """Lemma 2's 1/N: averaging N independently rounded copies divides the
    quantization variance by N."""
    d = 20000
    rng = np.random.default_rng(6)
    g = rng.uniform(-0.5, 0.5, size=d).astype(np.float32)
    P = uniform_params(0.5, 3)
    mse = {}
    for N in (1, 4, 16):
        pays = [O.compress(g, P, 77, i, 0) for i in range(N)]
        out = O.decompress_aggregate(pays, [P] * N, d, 3)
        mse[N] = ((out.astype(np.float64) - g) ** 2).mean()
    width = 1.0 / 7
    assert mse[1] == pytest.approx(width ** 2 / 6, rel=0.05)
    assert mse[4] == pytest.approx(mse[1] / 4, rel=0.08)
    assert mse[16] == pytest.approx(mse[1] / 16, rel=0.08)


def test_bf16_input_is_widened_exactly():
    rng = np.random.default_rng(8)
    x = (rng.standard_normal(4000) * 0.2).astype(np.float32)
    bits16 = (x.view(np.uint32) >> 16).astype(np.uint16)
    widened = (bits16.astype(np.uint32) << 16).view(np.float32)
    P = uniform_params(0.4, 2)
    assert (O.compress(bits16, P, 1, 2, 3) == O.compress(widened, P, 1, 2, 3)).all()
    sa, sb = O.stats(bits16), O.stats(widened)
    assert sa.tobytes() == sb.tobytes()
