"""Pins for the parameter design (Sec. IV) in oracle/params.py.

The closed forms below are consequences of the paper's boxed equations for a
pure symmetric power law p(g) = rho (gamma-1) g_min^(gamma-1) |g|^-gamma on
|g| > g_min with all mass in the tail (2 rho = 1); each is derived in the
docstring of its test.  The histogram handed to the oracle is the *analytic*
bin mass of that law, so the only slack is the piecewise-constant density
inside a bin (relative width 1/16 .. 1/32).
"""
import numpy as np
import pytest

from oracle import binding as O
from oracle import params as OP


def pareto_stats(gamma, x_min, absmax, n=1e12, g_min=None):
    """Expected histogram of |g| for the pure power law, as a stats-like mapping."""
    lo, hi = OP.bin_edges(absmax)
    sf = lambda t: np.where(t > x_min, (np.maximum(t, x_min) / x_min) ** -(gamma - 1), 1.0)
    hi_eff = np.minimum(hi, absmax)
    lo_eff = np.minimum(lo, absmax)
    mass = sf(lo_eff) - sf(hi_eff)
    mass[np.argmax(hi >= absmax)] += sf(np.array(absmax))        # fold the far tail into the top bin
    S = {"hist": n * mass, "absmax": absmax, "g_min": 0.0, "n_tail": 0, "sum_log_tail": 0.0}
    if g_min is not None:
        # exact terms: n_tail = n P(|g| > g_min), E ln(g/g_min | g > g_min) = 1/(gamma-1)
        S["g_min"] = g_min
        S["n_tail"] = n * float(sf(np.array(g_min)))
        S["sum_log_tail"] = S["n_tail"] / (gamma - 1)
    return S


X_MIN = 1e-4
X_EDGE = 2.0 ** -13        # a power-law edge that is also a bin edge: no half-filled bin
CASES_U = [(3.0, 3), (3.0, 2), (2.5, 2), (2.5, 4), (2.2, 3), (2.1, 2), (4.0, 3), (5.0, 3)]


@pytest.mark.parametrize("gamma,bits", CASES_U)
def test_uniform_alpha_closed_form(gamma, bits):
    """Sec. IV-A boxed equation with Q_U(alpha) = 1 - (alpha/g_min)^-(gamma-1) (all mass
    in the tail, 2 rho = 1): z = (alpha/g_min)^(gamma-1) solves z = C z/(z-1) with
    C = s^2/(gamma-2), so alpha* = g_min (1 + s^2/(gamma-2))^(1/(gamma-1)), and the
    truncated share of elements is 1/z = 1/(1+C)."""
    s = 2 ** bits - 1
    S = pareto_stats(gamma, X_MIN, absmax=X_MIN * 1e5, g_min=X_MIN)
    P = OP.tq_params_one(S, bits, O.GRID_UNIFORM)
    want = X_MIN * (1 + s * s / (gamma - 2)) ** (1 / (gamma - 1))
    assert float(P["alpha"]) == pytest.approx(want, rel=2e-3)
    assert float(P["gamma_hat"]) == pytest.approx(gamma, rel=1e-6)
    assert float(P["rho_hat"]) == pytest.approx(0.5, rel=1e-6)
    assert int(P["flags"]) == 0
    dens = OP.Density(S["hist"], S["absmax"])
    assert 1 - dens.Q_U(float(P["alpha"])) == pytest.approx(1 / (1 + s * s / (gamma - 2)), rel=2e-2)


def test_uniform_alpha_worked_value_config1():
    """gamma = 3, s = 7, x_min = 1e-4: alpha* = 1e-4 sqrt(50)."""
    S = pareto_stats(3.0, 1e-4, absmax=1.0, g_min=1e-4)
    assert float(OP.tq_params_one(S, 3, O.GRID_UNIFORM)["alpha"]) == pytest.approx(7.0710678e-4, rel=2e-3)


@pytest.mark.parametrize("t", [1.0, 1.5, 3.0])
def test_alpha_does_not_depend_on_where_in_the_tail_g_min_sits(t):
    """Scale invariance of the power law: g_min -> t g_min gives rho -> rho t^-(gamma-1),
    and g_min^(gamma-1) rho is unchanged, so the boxed equation has the same solution."""
    gamma, bits = 3.5, 3
    base = OP.tq_params_one(pareto_stats(gamma, X_MIN, 10.0, g_min=X_MIN), bits, O.GRID_UNIFORM)
    other = OP.tq_params_one(pareto_stats(gamma, X_MIN, 10.0, g_min=t * X_MIN), bits, O.GRID_UNIFORM)
    assert float(other["alpha"]) == pytest.approx(float(base["alpha"]), rel=1e-5)
    assert float(other["rho_hat"]) == pytest.approx(0.5 * t ** -(gamma - 1), rel=1e-6)


def y_star_nonuniform(gamma, s):
    """Sec. IV-B second boxed equation on the pure power law.  With y = alpha/g_min and
    I(y) = int_1^y t^(-gamma/3) dt one gets Q_N = 2 rho (gamma-1) I^3 / y^2, and the
    fixed point reads y^(gamma-3) I(y)^3 = K, K = s^2/((gamma-2)(gamma-1)).
    gamma = 3: (ln y)^3 = K.  Otherwise, with a = (gamma-3)/3: (y^a - 1)/a = K^(1/3)."""
    K = s * s / ((gamma - 2) * (gamma - 1))
    if gamma == 3.0:
        return np.exp(K ** (1 / 3))
    a = (gamma - 3) / 3
    base = 1 + a * K ** (1 / 3)
    return base ** (1 / a) if base > 0 else np.inf


@pytest.mark.parametrize("gamma,bits", [(3.0, 3), (3.0, 2), (4.0, 3), (3.5, 3), (5.0, 3), (2.5, 2), (4.0, 4)])
def test_nonuniform_alpha_closed_form(gamma, bits):
    s = 2 ** bits - 1
    S = pareto_stats(gamma, X_EDGE, absmax=X_EDGE * 1e6, g_min=X_EDGE)
    P = OP.tq_params_one(S, bits, O.GRID_NONUNIFORM)
    want = X_EDGE * y_star_nonuniform(gamma, s)
    assert float(P["alpha"]) == pytest.approx(want, rel=1e-3)
    assert int(P["flags"]) == 0
    # Sec. IV-B, closing remark: the non-uniform threshold is the larger one
    PU = OP.tq_params_one(S, bits, O.GRID_UNIFORM)
    assert float(P["alpha"]) > float(PU["alpha"])


def test_nonuniform_worked_values():
    assert y_star_nonuniform(3.0, 7) == pytest.approx(18.2542, rel=1e-4)
    assert y_star_nonuniform(4.0, 7) == pytest.approx(4.66805, rel=1e-4)


@pytest.mark.parametrize("gamma,bits", [(2.2, 3), (2.1, 2)])
def test_nonuniform_alpha_has_no_fixed_point_for_very_heavy_tails(gamma, bits):
    """For gamma < 3 the equation (y^a - 1)/a = K^(1/3), a < 0, has no solution once
    |a| K^(1/3) >= 1: the iteration runs away and is clamped at max|g| (no truncation)."""
    s = 2 ** bits - 1
    assert y_star_nonuniform(gamma, s) == np.inf
    S = pareto_stats(gamma, X_MIN, absmax=X_MIN * 1e4, g_min=X_MIN)
    P = OP.tq_params_one(S, bits, O.GRID_NONUNIFORM)
    assert float(P["alpha"]) == np.float32(S["absmax"])
    assert int(P["flags"]) & OP.FLAG_ALPHA_CLAMPED_MAX


@pytest.mark.parametrize("gamma,bits", [(3.0, 3), (3.0, 2), (4.0, 3), (2.5, 4)])
def test_nonuniform_levels_follow_the_cube_root_density(gamma, bits):
    """Sec. IV-B first boxed equation: lambda_s ~ p^(1/3).  With int_{-alpha}^{l_k} lambda_s = k
    and p ~ |g|^-gamma above g_min, the positive levels (k > s/2) satisfy
    l_k^(1-gamma/3) = g^(1-gamma/3) + ((2k-s)/s)(alpha^(1-gamma/3) - g^(1-gamma/3));
    for gamma = 3 this is the geometric grid l_k = g (alpha/g)^((2k-s)/s)."""
    s = 2 ** bits - 1
    S = pareto_stats(gamma, X_EDGE, absmax=1.0, g_min=X_EDGE)
    alpha = 20 * X_EDGE
    P = OP.tq_params_one(S, bits, O.GRID_NONUNIFORM, alpha_override=alpha)
    lv = P["level"][: s + 1].astype(np.float64)
    assert lv[0] == -np.float32(alpha) and lv[s] == np.float32(alpha)
    assert (lv == -lv[::-1]).all() and (np.diff(lv) > 0).all()
    for k in range((s + 1) // 2, s):
        f = (2 * k - s) / s
        if gamma == 3.0:
            want = X_EDGE * (alpha / X_EDGE) ** f
        else:
            e = 1 - gamma / 3
            want = (X_EDGE ** e + f * (alpha ** e - X_EDGE ** e)) ** (1 / e)
        assert lv[k] == pytest.approx(want, rel=2e-3)
    # inverse widths are what they say
    assert np.allclose(P["inv_w"][:s], 1 / np.diff(lv), rtol=1e-6)
    # and more points sit where the density is high: cells widen away from zero
    w = np.diff(lv)[(s + 1) // 2:]
    assert (np.diff(w) > 0).all()


def test_density_integrates_to_s():
    """Sec. III-A: int lambda_s = s, i.e. the mass of p^(1/3) between consecutive levels is
    the same for every cell -- checked on a sampled, non-power-law histogram."""
    rng = np.random.default_rng(0)
    g = np.concatenate([rng.standard_normal(200000) * 1e-3, rng.standard_t(2.5, 100000) * 3e-3]).astype(np.float32)
    S = O.stats(g)[0]
    alpha = 0.01
    P = OP.tq_params_one(S, 3, O.GRID_NONUNIFORM, alpha_override=alpha)
    dens = OP.Density(S["hist"], S["absmax"])
    lv = P["level"][:8].astype(np.float64)
    G = np.sign(lv) * np.array([dens.half_int_p13(abs(x)) for x in lv])
    cell = np.diff(G)
    assert np.allclose(cell, cell.mean(), rtol=1e-4)


def test_uniform_levels_definition():
    """Sec. IV-A: L = {-alpha + k 2 alpha/s}."""
    for bits, alpha in [(2, 0.3), (3, 7.07e-4), (4, 123.0)]:
        s = 2 ** bits - 1
        S = pareto_stats(3.0, X_MIN, 1e3)
        P = OP.tq_params_one(S, bits, O.GRID_UNIFORM, alpha_override=alpha)
        a = float(np.float32(alpha))
        lv = P["level"][: s + 1].astype(np.float64)
        assert lv[0] == -a and lv[s] == a
        assert np.allclose(lv, -a + np.arange(s + 1) * 2 * a / s, rtol=0, atol=a * 2.0 ** -23)
        assert np.allclose(P["inv_w"][:s], s / (2 * a), rtol=2.0 ** -23)
        assert (P["inv_w"][s:] == 0).all() and (P["level"][s + 1:] == 0).all()


def test_holder_ordering_of_QN_and_QU():
    """Sec. IV-B: Q_N(alpha) <= Q_U(alpha) <= 1 for any density and alpha."""
    rng = np.random.default_rng(1)
    for trial in range(20):
        hist = np.zeros(O.NBINS)
        idx = rng.integers(1, O.NBINS - 1, size=rng.integers(1, 60))
        hist[idx] = rng.integers(1, 10 ** 6, size=idx.size)
        dens = OP.Density(hist, 1e6)
        for alpha in np.exp(rng.uniform(np.log(1e-12), np.log(1e5), size=10)):
            qn, qu = dens.Q_N(alpha), dens.Q_U(alpha)
            assert qn <= qu * (1 + 1e-12) and qu <= 1 + 1e-12


@pytest.mark.parametrize("gamma,bits", [(4.0, 3), (3.5, 2), (5.0, 4)])
def test_fixed_point_nearly_minimises_the_error_model(gamma, bits):
    """Sec. IV-A: the boxed alpha is the stationary point of
    E(alpha) = Q_U(alpha) alpha^2/s^2 + 4 rho g_min^(gamma-1) alpha^(3-gamma)/((gamma-2)(gamma-3))
    with Q_U held fixed.  Brute force over a fine grid: alpha within 10 % of the arg min and
    the error within 1 % of the minimum."""
    s = 2 ** bits - 1
    S = pareto_stats(gamma, X_MIN, 1.0, g_min=X_MIN)
    dens = OP.Density(S["hist"], S["absmax"])
    E = lambda a: dens.Q_U(a) * a * a / (s * s) + 4 * 0.5 * X_MIN ** (gamma - 1) * a ** (3 - gamma) / ((gamma - 2) * (gamma - 3))
    grid = X_MIN * np.exp(np.linspace(np.log(1.01), np.log(200), 4000))
    vals = np.array([E(a) for a in grid])
    a_star = float(OP.tq_params_one(S, bits, O.GRID_UNIFORM)["alpha"])
    assert a_star == pytest.approx(grid[vals.argmin()], rel=0.10)
    assert E(a_star) <= vals.min() * 1.01


def test_formula_alpha_is_near_the_brute_force_optimum_on_a_small_sample():
    """End to end on 20000 sampled values (gamma = 4): the expected squared error of
    Q[T_alpha(g)], computed exactly per element as (x-l)(u-x) inside and (|x|-alpha)^2
    outside, at the formula's alpha is within 10 % of the best alpha found by grid search."""
    rng = np.random.default_rng(2)
    gamma, bits = 4.0, 3
    s = 7
    g = (X_MIN * rng.uniform(size=20000) ** (-1 / (gamma - 1)) * rng.choice([-1.0, 1.0], size=20000)).astype(np.float32)
    S = O.stats(g, g_min=X_MIN)[0]
    P = OP.tq_params_one(S, bits, O.GRID_UNIFORM)
    x = np.abs(g.astype(np.float64))

    def err(alpha):
        xc = np.minimum(x, alpha)
        step = 2 * alpha / s
        t = (xc + alpha) / step
        k = np.minimum(np.floor(t), s - 1)
        lo = -alpha + k * step
        return ((xc - lo) * (lo + step - xc)).sum() + ((x - xc) ** 2).sum()

    grid = X_MIN * np.linspace(1.05, 12, 600)
    best = min(err(a) for a in grid)
    assert err(float(P["alpha"])) <= 1.10 * best
    # without truncation (alpha = max|g|) the error is far worse: the paper's motivation
    assert err(float(S["absmax"])) > 3 * best


def test_binned_tail_index_is_close_to_the_exact_one():
    """Automatic g_min: gamma from bin counts (bins at their geometric mean) against the exact
    maximum-likelihood value from the analytic tail; the binning bias is O(w^2), w = ln2/16."""
    for gamma in (2.5, 3.0, 4.0):
        S = pareto_stats(gamma, X_MIN, 1e3)
        P = OP.tq_params_one(S, 3, O.GRID_UNIFORM)
        assert float(P["gamma_hat"]) == pytest.approx(gamma, rel=2e-3)
        lo, _ = OP.bin_edges(1.0)
        assert float(P["g_min"]) in lo.astype(np.float32)
        # 0.9-quantile of |g|: (g_min/x_min)^-(gamma-1) ~ 0.1, from above, within a bin
        tail = (float(P["g_min"]) / X_MIN) ** -(gamma - 1)
        assert 0.1 <= tail < 0.1 * (1 + 1 / 16) ** (gamma - 1) * 1.001
        assert float(P["rho_hat"]) == pytest.approx(tail / 2, rel=1e-3)
        # same threshold as with the exact tail terms
        PE = OP.tq_params_one(pareto_stats(gamma, X_MIN, 1e3, g_min=X_MIN), 3, O.GRID_UNIFORM)
        assert float(P["alpha"]) == pytest.approx(float(PE["alpha"]), rel=5e-3)


def test_override_and_no_truncation_switch():
    S = pareto_stats(3.0, X_MIN, 0.37, g_min=X_MIN)
    P = OP.tq_params_one(S, 2, O.GRID_UNIFORM, alpha_override=-1.0)
    assert float(P["alpha"]) == np.float32(0.37) and int(P["flags"]) & OP.FLAG_ALPHA_OVERRIDE
    P = OP.tq_params_one(S, 2, O.GRID_UNIFORM, alpha_override=0.01)
    assert float(P["alpha"]) == np.float32(0.01)


def test_degenerate_inputs_give_usable_parameters():
    zeros = O.stats(np.zeros(256, dtype=np.float32))[0]
    for grid in (O.GRID_UNIFORM, O.GRID_NONUNIFORM):
        P = OP.tq_params_one(zeros, 3, grid)
        assert int(P["flags"]) & OP.FLAG_DEGENERATE and float(P["alpha"]) > 0
        assert np.isfinite(P["inv_w"]).all() and (np.diff(P["level"][:8]) > 0).all()
        # a threshold the caller gives is used even when there is nothing to design from
        P = OP.tq_params_one(zeros, 3, grid, alpha_override=0.5)
        assert float(P["alpha"]) == 0.5 and P["level"][0] == -0.5 and P["level"][7] == 0.5
        assert int(P["flags"]) & OP.FLAG_DEGENERATE and int(P["flags"]) & OP.FLAG_ALPHA_OVERRIDE
    const = O.stats(np.full(256, 0.25, dtype=np.float32))[0]       # one point mass
    for grid in (O.GRID_UNIFORM, O.GRID_NONUNIFORM):
        P = OP.tq_params_one(const, 2, grid)
        assert float(P["alpha"]) == 0.25 and np.isfinite(P["inv_w"]).all()
        assert (np.diff(P["level"][:4]) >= 0).all()
