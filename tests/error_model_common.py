"""Shared by the error-model tests (CPU oracle and GPU library): the synthetic heavy-tailed
sample, the expected squared error of a codebook on it, and the paper's model of that error."""
import numpy as np

GAMMA, X_MIN = 4.0, 1e-3          # inside the range 3 < gamma <= 5 the error model is stated for
SWEEP = (0.35, 0.5, 0.7, 1.0, 1.4, 2.0, 2.8)


def pareto_sample(d, seed):
    """Symmetric power law with density exponent GAMMA above X_MIN (Sec. IV-A), as float32."""
    rng = np.random.default_rng(seed)
    mag = X_MIN * rng.random(d) ** (-1.0 / (GAMMA - 1.0))
    return (mag * np.where(rng.random(d) < 0.5, -1.0, 1.0)).astype(np.float32)


def expected_mse(g, P):
    """Mean over the sample of E|Q[T_alpha(g)] - g|^2 for one parameter record P: the rounding
    variance (x - l)(u - x) of Lemma 1 inside [-alpha, alpha] plus the squared truncation
    error outside (Eq. 1)."""
    s = int(P["s"][0])
    lv = P["level"][0][: s + 1].astype(np.float64)
    a = float(P["alpha"][0])
    x = g.astype(np.float64)
    xc = np.clip(x, -a, a)
    k = np.clip(np.searchsorted(lv, xc, side="right") - 1, 0, s - 1)
    return float(np.mean((xc - lv[k]) * (lv[k + 1] - xc) + (x - xc) ** 2))


def model_uniform(g, P):
    """Per-element error of the truncated uniform quantizer as Sec. IV-A models it (the first
    displayed equation after the power-law tail density, with d = N = 1): Q_U alpha^2 / s^2
    plus the tail's truncation term."""
    a, s = float(P["alpha"][0]), int(P["s"][0])
    gam, rho, gmin = float(P["gamma_hat"][0]), float(P["rho_hat"][0]), float(P["g_min"][0])
    q_u = float(np.mean(np.abs(g) <= a))
    return q_u * a * a / s ** 2 + 4.0 * rho * gmin ** (gam - 1.0) * a ** (3.0 - gam) / ((gam - 2.0) * (gam - 3.0))
