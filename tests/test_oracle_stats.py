"""Pins for the statistics reductions (Sec. IV: rho, Q_U, integral of p^(1/3); Sec. V: MLE)."""
import numpy as np
import pytest

from oracle import binding as O
from oracle import params as OP


def test_bins_are_sixteenths_of_octaves_between_2pow_minus40_and_2pow16():
    lo, hi = OP.bin_edges(1.0)
    # edges by searching an explicitly built, sorted edge list (independent of bit tricks)
    edges = np.concatenate([[0.0], lo[1:], [np.inf]])
    rng = np.random.default_rng(0)
    xs = np.concatenate([
        np.exp(rng.uniform(np.log(1e-14), np.log(1e6), size=4000)),
        lo[1:], np.nextafter(lo[1:].astype(np.float32), np.float32(0)),   # at and just below edges
        [0.0, 2.0 ** -41, 2.0 ** -40, 65535.9, 65536.0, 3e38, 1e-45],
    ]).astype(np.float32)
    want = np.searchsorted(edges.astype(np.float64), xs.astype(np.float64), side="right") - 1
    got = np.array([O.bin_index(float(x)) for x in xs])
    assert (got == want).all()
    assert lo[1] == 2.0 ** -40 and hi[O.NBINS - 2] == 2.0 ** 16
    assert np.allclose(hi[1:-1] / lo[1:-1], 1 + 1 / (16 + (np.arange(896) % 16)))


def test_histogram_counts_extremes_and_nonfinite():
    rng = np.random.default_rng(1)
    n = 50000
    g = (1e-4 * rng.uniform(size=n) ** -0.5 * rng.choice([-1.0, 1.0], size=n)).astype(np.float32)
    g[[5, 77, 4000]] = [np.nan, np.inf, -np.inf]
    g[[6, 78]] = [0.0, -0.0]
    S = O.stats(g)[0]
    fin = np.isfinite(g)
    assert S["n"] == n and S["n_nonfinite"] == 3
    assert S["hist"].sum() == fin.sum()
    assert S["absmax"] == np.abs(g[fin]).max()
    lo, _ = OP.bin_edges(1.0)
    edges = np.concatenate([[0.0], lo[1:], [np.inf]])
    want, _ = np.histogram(np.abs(g[fin]).astype(np.float64), bins=edges)
    assert (S["hist"] == want).all()
    assert S["hist"][0] == 2 and S["n_tail"] == 0 and S["sum_log_tail"] == 0.0


def test_buckets_partition_the_tensor():
    rng = np.random.default_rng(2)
    d, B = 1000, 384
    g = rng.standard_normal(d).astype(np.float32)
    S = O.stats(g, bucket_elems=B, g_min=0.5)
    assert S.size == 3 and list(S["n"]) == [384, 384, 232]
    for j in range(3):
        one = O.stats(g[j * B:(j + 1) * B], g_min=0.5)[0]
        assert S[j].tobytes() == one.tobytes()


@pytest.mark.parametrize("gamma", [2.2, 3.0, 4.5])
def test_tail_terms_give_the_maximum_likelihood_tail_index(gamma):
    """Sec. V: gamma = 1 + n [sum ln(g_j/g_min)]^-1 over g_j > g_min.  On exact Pareto
    samples the estimator is consistent with standard error (gamma-1)/sqrt(n); the
    threshold can sit anywhere in the tail (scale invariance of the power law)."""
    rng = np.random.default_rng(3)
    n = 400000
    x_min = 1e-4
    g = (x_min * rng.uniform(size=n) ** (-1 / (gamma - 1)) * rng.choice([-1.0, 1.0], size=n)).astype(np.float32)
    for g_min in (x_min, 2.5 * x_min):
        S = O.stats(g, g_min=g_min)[0]
        n_tail = int(S["n_tail"])
        assert n_tail == int((np.abs(g) > np.float32(g_min)).sum())
        gamma_hat = 1 + n_tail / S["sum_log_tail"]
        assert abs(gamma_hat - gamma) < 4.5 * (gamma - 1) / np.sqrt(n_tail)
        # two-sided tail mass = (g_min/x_min)^-(gamma-1)
        assert n_tail / n == pytest.approx((g_min / x_min) ** -(gamma - 1), abs=4 / np.sqrt(n))
