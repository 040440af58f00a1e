"""Pins for the element-wise path of the oracle: Eq. (1), Eq. (2), Lemma 1, Alg. 1.

Nothing here re-types the oracle's formula: each test states a property the
paper or the mathematics fixes and checks the oracle's outputs against it.
"""
import numpy as np
import pytest

from oracle import binding as O
from oracle import params as OP

R_ALL = np.arange(65536)


def make_params(levels, grid, alpha=None):
    """PARAMS record with a hand-made codebook (widths inverted in fp64, rounded once)."""
    levels = np.asarray(levels, dtype=np.float32)
    s = levels.size - 1
    bits = {3: 2, 7: 3, 15: 4}[s]
    P = np.zeros(1, dtype=O.PARAMS_DTYPE)
    P["alpha"] = levels[-1] if alpha is None else alpha
    P["bits"], P["s"], P["grid"] = bits, s, grid
    P["level"][0, : s + 1] = levels
    if grid == O.GRID_UNIFORM:
        P["inv_w"][0, :s] = np.float32(s / (2.0 * float(P["alpha"][0])))
    else:
        width = np.diff(levels.astype(np.float64))
        # an empty cell has reciprocal 0, as the parameter record is specified
        P["inv_w"][0, :s] = np.where(width > 0, 1.0 / np.where(width > 0, width, 1.0), 0.0).astype(np.float32)
    return P


def uniform_params(alpha, bits):
    s = (1 << bits) - 1
    return make_params(OP.uniform_levels(np.float32(alpha), s), O.GRID_UNIFORM)


NONUNIFORM_7 = [-1.0, -0.45, -0.2, -0.05, 0.05, 0.2, 0.45, 1.0]
NONUNIFORM_3 = [-2.5e-3, -3e-4, 3e-4, 2.5e-3]


def all_outcomes(x, P):
    lv = P["level"][0]
    return np.array([lv[O.quantize_one(x, P, r)] for r in R_ALL], dtype=np.float64)


@pytest.mark.parametrize("P", [uniform_params(1.0, 2), uniform_params(7.07e-4, 3),
                               uniform_params(0.3, 4),
                               make_params(NONUNIFORM_7, O.GRID_NONUNIFORM),
                               make_params(NONUNIFORM_3, O.GRID_NONUNIFORM)])
def test_lemma1_unbiased_and_variance_by_enumeration(P):
    """Lemma 1: E[Q[g]] = g, and E|Q[g]-g|^2 = (g - l_{k-1})(l_k - g) <= |Delta_k|^2/4
    (appendix, proof of Lemma 1).  Enumerating every value of the 16-bit draw makes
    the expectation exact: the only slack is the 2^-16 grain of the probability."""
    s = int(P["s"][0])
    lv = P["level"][0, : s + 1].astype(np.float64)
    rng = np.random.default_rng(1)
    xs = list(rng.uniform(lv[0], lv[-1], size=6)) + [0.0, float(lv[1]) * 0.999]
    for x in xs:
        x = float(np.float32(x))
        k = int(np.searchsorted(lv, x, side="right")) - 1
        k = min(max(k, 0), s - 1)
        lo, hi = lv[k], lv[k + 1]
        out = all_outcomes(x, P)
        assert set(np.unique(out)) <= {lo, hi}          # only the cell's two ends occur
        width = hi - lo
        assert abs(out.mean() - x) <= width * 2.0 ** -16 + 1e-7 * abs(x)
        var = ((out - x) ** 2).mean()
        assert abs(var - (x - lo) * (hi - x)) <= width ** 2 * 2.0 ** -15
        assert var <= width ** 2 / 4 * (1 + 1e-6)


def test_lemma1_high_rate_mean_variance_is_width_squared_over_six():
    """Appendix, proof of Lemma 1, step (a): for g uniform in a cell the mean squared
    error is |Delta_k|^2 / 6."""
    P = make_params(NONUNIFORM_7, O.GRID_NONUNIFORM)
    lv = P["level"][0, :8].astype(np.float64)
    lo, hi = lv[5], lv[6]
    rng = np.random.default_rng(7)
    xs = rng.uniform(lo, hi, size=40000).astype(np.float32)
    r = rng.integers(0, 65536, size=xs.size)
    q = np.array([lv[O.quantize_one(float(x), P, int(rr))] for x, rr in zip(xs, r)])
    mse = ((q - xs) ** 2).mean()
    assert abs(mse / ((hi - lo) ** 2 / 6) - 1) < 0.03


@pytest.mark.parametrize("grid", [O.GRID_UNIFORM, O.GRID_NONUNIFORM])
def test_points_on_the_codebook_are_kept_exactly(grid):
    """Eq. (2) with g = l_k: p_r is 0 or 1, so the outcome is l_k whatever the draw."""
    if grid == O.GRID_UNIFORM:
        # levels exactly representable so that "on the grid" is exact: alpha = 3.5, s = 7
        P = uniform_params(3.5, 3)
    else:
        P = make_params(NONUNIFORM_7, O.GRID_NONUNIFORM)
    lv = P["level"][0, :8]
    for k, x in enumerate(lv):
        codes = {O.quantize_one(float(x), P, r) for r in (0, 1, 30000, 65534, 65535)}
        assert codes == {k}


@pytest.mark.parametrize("grid", [O.GRID_UNIFORM, O.GRID_NONUNIFORM])
def test_truncation_then_quantization_of_outliers(grid):
    """Eq. (1): |g| > alpha is cut to sgn(g) alpha, which is the end point of the codebook."""
    P = uniform_params(0.5, 3) if grid == O.GRID_UNIFORM else make_params(NONUNIFORM_7, grid)
    a = float(P["alpha"][0])
    s = int(P["s"][0])
    for r in (0, 12345, 65535):
        assert O.quantize_one(a * 1.0001, P, r) == s
        assert O.quantize_one(3e38, P, r) == s
        assert O.quantize_one(float("inf"), P, r) == s
        assert O.quantize_one(-a * 1.0001, P, r) == 0
        assert O.quantize_one(float("-inf"), P, r) == 0
        # NaN is encoded like +0: the two levels around zero
        assert O.quantize_one(float("nan"), P, r) == O.quantize_one(0.0, P, r)
    assert O.truncate(0.3, 0.5) == pytest.approx(0.3)
    assert O.truncate(-0.7, 0.5) == -0.5 and O.truncate(0.7, 0.5) == 0.5
    assert O.truncate(0.5, 0.5) == 0.5 and O.truncate(-0.0, 0.5) == 0.0


def test_code_is_monotone_in_g_and_in_the_draw():
    """For a fixed draw the code cannot decrease when g grows (both grids)."""
    for P in (uniform_params(1.0, 4), make_params(NONUNIFORM_7, O.GRID_NONUNIFORM)):
        xs = np.linspace(-1.2, 1.2, 2001).astype(np.float32)
        for r in (0, 9000, 40000, 65535):
            c = np.array([O.quantize_one(float(x), P, r) for x in xs])
            assert (np.diff(c) >= 0).all() and c.min() == 0 and c.max() == int(P["s"][0])
        # and for fixed g a larger draw can only push the code up
        c = np.array([O.quantize_one(0.1234, P, r) for r in range(0, 65536, 97)])
        assert (np.diff(c) >= 0).all()


def test_truncation_bias_of_a_power_law_tail_matches_the_closed_form():
    """Sec. IV-A, second term of the truncated-quantization error:
    2 int_alpha^inf (g-alpha)^2 p(g) dg = 4 rho g_min^(gamma-1) alpha^(3-gamma) /
    ((gamma-2)(gamma-3)) for p = rho (gamma-1) g_min^(gamma-1) |g|^-gamma.
    The integral of (g - T_alpha[g])^2 p(g) is taken by quadrature on a log grid with
    T_alpha evaluated by the oracle."""
    for gamma, g_min, rho, y in [(4.0, 1e-3, 0.5, 3.0), (3.5, 2e-4, 0.2, 5.0), (5.0, 1.0, 0.35, 1.7)]:
        alpha = np.float32(y * g_min)
        t = np.exp(np.linspace(np.log(float(alpha)), np.log(float(alpha) * 1e12), 40001))
        Tt = np.array([O.truncate(float(np.float32(v)), float(alpha)) for v in t])
        f = (t - Tt) ** 2 * rho * (gamma - 1) * g_min ** (gamma - 1) * t ** -gamma
        integral = 2 * np.sum(0.5 * (f[1:] + f[:-1]) * np.diff(t))
        closed = 4 * rho * g_min ** (gamma - 1) * float(alpha) ** (3 - gamma) / ((gamma - 2) * (gamma - 3))
        assert integral == pytest.approx(closed, rel=1e-3)
        # and inside [-alpha, alpha] truncation changes nothing
        for v in np.linspace(-float(alpha), float(alpha), 11):
            v = float(np.float32(v))
            assert O.truncate(v, float(alpha)) == v


def test_total_error_matches_variance_plus_bias_decomposition():
    """Appendix, proof of Lemma 2, first display: E|Q[T(g)] - g|^2 = quantization
    variance + truncation bias.  Empirical MSE over many steps on a small Pareto
    sample against sum over samples of (x-l)(u-x) inside and (|x|-alpha)^2 outside,
    and against the bound sum P_k |Delta_k|^2 / 4 + bias (Lemma 1)."""
    rng = np.random.default_rng(3)
    n = 4096
    g = (1e-4 * rng.uniform(size=n) ** -0.5 * rng.choice([-1.0, 1.0], size=n)).astype(np.float32)
    alpha = np.float32(7.07e-4)
    for P in (uniform_params(alpha, 3),
              make_params(np.float32(alpha) * np.array(NONUNIFORM_7), O.GRID_NONUNIFORM)):
        s = int(P["s"][0])
        lv = P["level"][0, : s + 1].astype(np.float64)
        steps = 200
        err2 = np.zeros(n)
        for step in range(steps):
            payload = O.compress(g, P, seed=99, worker=0, step=step)
            q = O.dequantize(payload, P, n, int(P["bits"][0]))
            err2 += (q.astype(np.float64) - g) ** 2
        mse = err2.sum() / steps
        gc = np.clip(g.astype(np.float64), -float(alpha), float(alpha))
        k = np.clip(np.searchsorted(lv, gc, side="right") - 1, 0, s - 1)
        var = (gc - lv[k]) * (lv[k + 1] - gc)
        bias = (np.abs(g.astype(np.float64)) - np.abs(gc)) ** 2
        # unbiased inside, deterministic clipping outside: cross term vanishes
        assert mse == pytest.approx((var + bias).sum(), rel=0.03)
        bound = ((lv[k + 1] - lv[k]) ** 2 / 4 + bias).sum()
        assert mse <= bound


def test_mean_over_steps_converges_to_the_truncated_gradient():
    """Unbiasedness through the whole compress -> dequantize path (Lemma 1, Alg. 1)."""
    rng = np.random.default_rng(5)
    n = 2000
    g = rng.standard_normal(n).astype(np.float32) * 0.3
    P = uniform_params(0.5, 2)
    acc = np.zeros(n)
    M = 400
    for step in range(M):
        acc += O.dequantize(O.compress(g, P, 1, 3, step), P, n, 2)
    mean = acc / M
    width = 1.0 / 3
    sigma = width / 2 / np.sqrt(M)
    assert np.abs(mean - np.clip(g, -0.5, 0.5)).max() < 5 * sigma


@pytest.mark.parametrize("P", [make_params(NONUNIFORM_7, O.GRID_NONUNIFORM),
                               make_params(NONUNIFORM_3, O.GRID_NONUNIFORM),
                               make_params([-0.05, -0.01, 0.02, 0.05], O.GRID_NONUNIFORM),
                               make_params([-1.0, -0.5, 0.0, 0.5, 0.5, 0.75, 1.0, 1.0], O.GRID_NONUNIFORM),
                               make_params([-1.0, -1.0 + 2.0 ** -23, 0.0, 1.0], O.GRID_NONUNIFORM)])
def test_on_a_level_table_truncation_changes_the_code_only_through_an_empty_first_cell(P):
    """Eq. (1) followed by Eq. (2) on a level table whose first cell is not empty: beyond +alpha the
    cell is the last one and p_r is at least 1 (or 0 for an empty last cell), below -alpha it is the
    first one and p_r is below 0, so the code is the end level for every draw whether or not the value
    was truncated first.  (The GPU kernel's level-table path relies on this: it writes the
    truncation out only for codebooks with l_1 = l_0.)  Checked by enumerating all draws with the
    truncation switched off -- the same codebook under a threshold nothing exceeds."""
    free = P.copy()
    free["alpha"] = np.float32(3.4e38)
    a = float(P["alpha"][0])
    s = int(P["s"][0])
    lv = P["level"][0, : s + 1]
    assert lv[1] > lv[0]
    xs = [a, np.nextafter(np.float32(a), np.float32(np.inf)), 1.5 * a, 100 * a, 3.0e38, np.inf,
          -a, np.nextafter(np.float32(-a), np.float32(-np.inf)), -1.5 * a, -3.0e38, -np.inf]
    xs += [float(l) for l in lv] + [0.0, 0.3 * a, -0.7 * a]
    for x in xs:
        with_t = O.enumerate_draws(np.float32(x), P, eq2=True)
        without = O.enumerate_draws(np.float32(x), free, eq2=True)
        assert (with_t == without).all(), (float(x), with_t[: s + 1], without[: s + 1])
    # ... and the exception: an empty first cell, a value below -alpha
    E = make_params([-1.0, -1.0, 0.0, 1.0], O.GRID_NONUNIFORM)
    F = E.copy()
    F["alpha"] = np.float32(3.4e38)
    assert O.quantize_eq2(-2.0, E, 7) == 1 and O.quantize_eq2(-2.0, F, 7) == 0
