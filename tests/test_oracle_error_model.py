"""The paper's central claims on synthetic heavy-tailed data, on the CPU oracle: the error of
the truncated quantizer is what Lemma 1 plus Eq. (1) predict, Sec. IV-A's model bounds it,
truncating at the formula's alpha beats not truncating (QSGD / NQSGD), the formula's alpha
is close to the best of a sweep, and the non-uniform codebook of Sec. IV-B beats the uniform
one at equal bits."""
import numpy as np
import pytest

from oracle import binding as O
from oracle import params as OP
from error_model_common import SWEEP, X_MIN, expected_mse, model_uniform, pareto_sample

D = 1 << 17


@pytest.fixture(scope="module")
def sample():
    g = pareto_sample(D, 11)
    return g, O.stats(g, bucket_elems=0, g_min=X_MIN)


def roundtrip_mse(g, P, bits):
    pay = O.compress(g, P, 7, 0, 0, bucket_elems=0)
    out = O.decompress_aggregate([pay], [P], g.size, bits, bucket_elems=0)
    return float(np.mean((out.astype(np.float64) - g.astype(np.float64)) ** 2))


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("grid", [0, 1, 2])
def test_empirical_error_is_the_expected_one(sample, bits, grid):
    g, S = sample
    P = OP.tq_params(S, bits, grid)
    assert abs(roundtrip_mse(g, P, bits) / expected_mse(g, P) - 1.0) < 0.02


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_model_of_sec_4a_bounds_the_uniform_error(sample, bits):
    g, S = sample
    P = OP.tq_params(S, bits, 0)
    e, m = expected_mse(g, P), model_uniform(g, P)
    assert 0.5 * m < e < 1.05 * m           # the model charges Delta^2/4 per element, Lemma 1's bound


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("grid", [0, 1, 2])
def test_truncation_helps_and_formula_alpha_is_near_the_best(sample, bits, grid):
    g, S = sample
    P = OP.tq_params(S, bits, grid)
    e = expected_mse(g, P)
    no_trunc = expected_mse(g, OP.tq_params(S, bits, grid, -1.0))       # alpha = max|g|
    # the non-uniform codebook already spends few levels on the far tail, so its gain is small
    assert e < no_trunc / (20.0 if grid == 0 else 1.0)
    a = float(P["alpha"][0])
    sweep = [expected_mse(g, OP.tq_params(S, bits, grid, a * f)) for f in SWEEP]
    # the appendix calls the BiScaled alpha a one-step approximation: a wider margin there
    assert e <= (1.2 if grid < 2 else 1.4) * min(sweep)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_nonuniform_codebook_beats_uniform(sample, bits):
    g, S = sample
    assert expected_mse(g, OP.tq_params(S, bits, 1)) < expected_mse(g, OP.tq_params(S, bits, 0))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_biscaled_codebook_beats_uniform(sample, bits):
    """The closing claim of the BiScaled appendix."""
    g, S = sample
    assert expected_mse(g, OP.tq_params(S, bits, 2)) < expected_mse(g, OP.tq_params(S, bits, 0))
