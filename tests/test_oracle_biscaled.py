"""Pins for the truncated BiScaled quantizer (appendix "Truncated BiScaled Quantization")
in oracle/params.py: closed forms on densities for which the appendix's quantities are
known, Hoelder's inequality between the three Q's, the structure of the codebook, a brute
force over all (beta, s_beta), and the boxed fixed point."""
import numpy as np
import pytest

from oracle import binding as O
from oracle import params as OP
from test_oracle_params import pareto_stats

NB = O.NBINS


def two_level_density(beta_edge, alpha_edge, p1, p2, n=1e12):
    """Histogram of a symmetric density that is p1 on |g| < lo[beta_edge] and p2 up to
    lo[alpha_edge] (both bin edges), zero beyond; returns (Density, beta, alpha)."""
    lo, hi = OP.bin_edges(1.0)
    mass = np.zeros(NB)
    mass[:beta_edge] = 2 * p1 * (hi - lo)[:beta_edge]
    mass[beta_edge:alpha_edge] = 2 * p2 * (hi - lo)[beta_edge:alpha_edge]
    return OP.Density(n * mass / mass.sum(), lo[alpha_edge]), lo[beta_edge], lo[alpha_edge]


def test_q_b_of_a_flat_density_does_not_depend_on_k():
    """p constant on [-A, A]: 2 int_0^{kA} p = k and 2 int_{kA}^{A} p = 1 - k, so
    Q_B = [(1-k)^(1/3) (1-k)^(2/3) + k^(1/3) k^(2/3)]^3 = 1 = Q_U(A) for every k."""
    dens, _, A = two_level_density(600, 700, 1.0, 1.0)
    for k in (0.0, 0.1, 0.37, 0.5, 0.9, 1.0):
        assert dens.Q_B(A, k) == pytest.approx(1.0, rel=1e-12)
    for k in (0.2, 0.6):                     # and inside the support, Q_B = Q_U(alpha) = alpha / A
        assert dens.Q_B(0.5 * A, k) == pytest.approx(0.5, rel=1e-12)


@pytest.mark.parametrize("ratio", [8.0, 64.0, 0.125])
def test_two_level_density_is_recovered(ratio):
    """For a density with two plateaus the BiScaled family contains the optimal density
    lambda ~ p^(1/3) of Sec. IV-B, so min_k Q_B(alpha, k) = Q_N(alpha), attained at the true
    breakpoint; Hoelder's inequality puts every other k in between Q_N and Q_U."""
    dens, beta, alpha = two_level_density(640, 720, ratio, 1.0)
    j, q = dens.best_k(alpha)
    assert j == 640 and dens.lo[j] == beta
    assert q == pytest.approx(dens.Q_N(alpha), rel=1e-12)
    for jj in range(560, 720, 7):
        qq = dens.Q_B(alpha, dens.lo[jj] / alpha)
        assert dens.Q_N(alpha) * (1 - 1e-12) <= qq <= dens.Q_U(alpha) * (1 + 1e-12)
    # the share of cells the appendix's formula gives the inner region is the share of
    # int lambda_s that the optimal density of Sec. IV-B puts there
    s = 15
    k = beta / alpha
    c1, c2 = np.cbrt(ratio), 1.0
    share = c1 * k / (c2 * (1 - k) + c1 * k)
    assert share == pytest.approx(dens.half_int_p13(beta) / dens.half_int_p13(alpha), rel=1e-12)
    b, s_beta = OP.biscaled_split(dens, np.float32(alpha), s)
    assert b == beta and s_beta % 2 == 1 and abs(s_beta - s * share) <= 1.0 + 1e-9


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_hoelder_chain_on_a_power_law(bits):
    S = pareto_stats(3.5, 1e-4, absmax=1.0, g_min=1e-4)
    dens = OP.Density(S["hist"], S["absmax"])
    for a in (3e-4, 1e-3, 7e-3):
        _, q = dens.best_k(a)
        assert dens.Q_N(a) * (1 - 1e-12) <= q <= dens.Q_U(a) * (1 + 1e-12) <= 1 + 1e-12
    # smaller Q => larger threshold (the appendix's closing remark)
    a_u = float(OP.tq_params_one(S, bits, O.GRID_UNIFORM)["alpha"])
    a_b = float(OP.tq_params_one(S, bits, O.GRID_BISCALED)["alpha"])
    a_n = float(OP.tq_params_one(S, bits, O.GRID_NONUNIFORM)["alpha"])
    assert a_u <= a_b * (1 + 1e-6) and a_b <= a_n * (1 + 1e-6)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("gamma", [3.5, 4.5])
def test_boxed_fixed_point_and_codebook_structure(bits, gamma):
    s = 2 ** bits - 1
    S = pareto_stats(gamma, 1e-4, absmax=1.0, g_min=1e-4)
    P = OP.tq_params_one(S, bits, O.GRID_BISCALED)
    dens = OP.Density(S["hist"], S["absmax"])
    a = float(P["alpha"])
    assert int(P["flags"]) == 0
    _, q = dens.best_k(a)
    rhs = 1e-4 * (2 * 0.5 * s * s / ((gamma - 2) * q)) ** (1 / (gamma - 1))
    assert a == pytest.approx(rhs, rel=1e-6)                 # float32 rounding of alpha
    lv = P["level"][: s + 1].astype(np.float64)
    beta, s_beta = OP.biscaled_split(dens, P["alpha"], s)
    assert lv[0] == -a and lv[s] == a and (np.diff(lv) > 0).all()
    assert np.array_equal(lv, -lv[::-1])                     # symmetric
    h = (s - s_beta) // 2
    assert s_beta % 2 == 1 and 1 <= s_beta <= s - 2
    assert lv[h] == pytest.approx(-beta, rel=1e-7) and lv[h + s_beta] == pytest.approx(beta, rel=1e-7)
    assert np.allclose(np.diff(lv[h: h + s_beta + 1]), 2 * beta / s_beta, rtol=1e-5)
    assert np.allclose(np.diff(lv[h + s_beta:]), (a - beta) / h, rtol=1e-5)
    # int lambda_s = s: s_beta cells inside, s - s_beta outside
    iw = P["inv_w"][:s].astype(np.float64)
    assert np.allclose(iw * np.diff(lv), 1.0, rtol=1e-6)


@pytest.mark.parametrize("bits", [3, 4])
def test_choice_is_near_the_brute_force_minimum_of_the_appendix_model(bits):
    """At the designed alpha, the appendix's error model 2 p1 beta^3 / s_beta^2 +
    2 p2 (alpha-beta)^3 / s_alpha^2 (d = N = 1; the truncation term does not depend on the
    split) is evaluated for every edge beta and every odd s_beta; the design's pair must be
    within 25 % of the best (it rounds s_beta and takes one alternating step)."""
    s = 2 ** bits - 1
    S = pareto_stats(3.5, 1e-4, absmax=1.0, g_min=1e-4)
    dens = OP.Density(S["hist"], S["absmax"])
    P = OP.tq_params_one(S, bits, O.GRID_BISCALED)
    a = float(P["alpha"])

    def model(beta, s_beta):
        c_b, c_a = dens.Q_U(beta), dens.Q_U(a)
        p1, p2 = c_b / (2 * beta), (c_a - c_b) / (2 * (a - beta))
        return 2 * p1 * beta ** 3 / s_beta ** 2 + 2 * p2 * (a - beta) ** 3 / (s - s_beta) ** 2

    best = min(model(dens.lo[j], sb) for j in range(1, NB) if dens.lo[j] < a for sb in range(1, s - 1, 2))
    beta, s_beta = OP.biscaled_split(dens, P["alpha"], s)
    assert model(beta, s_beta) <= 1.25 * best


def test_no_edge_below_alpha_means_a_uniform_codebook():
    dens, _, _ = two_level_density(1, 2, 1.0, 1.0)            # all mass below 2^-40
    assert dens.best_k(2.0 ** -41)[0] == 0
    lv = OP.biscaled_levels(dens, np.float32(2.0 ** -41), 7)
    assert np.allclose(np.diff(lv.astype(np.float64)), 2 * 2.0 ** -41 / 7, rtol=1e-6)
