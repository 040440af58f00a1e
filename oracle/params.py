"""Parameter design of the truncated quantizer in fp64 -- TEST INFRASTRUCTURE.

Plain numpy statement of Sec. IV of arXiv 2402.01798 ("Optimal Quantizer
Parameter Design") fed by the per-bucket statistics of ``tq_oracle.c``:

* tail index by maximum likelihood (Sec. V):  gamma = 1 + n / sum_j ln(g_j / g_min)
* one-sided tail mass (Sec. IV-A, below the power-law model):  rho = P(g > g_min)
* truncation threshold, uniform grid (Sec. IV-A, boxed equation):
      alpha = g_min * [2 rho s^2 / ((gamma - 2) Q_U(alpha))]^(1/(gamma-1)),
      Q_U(alpha) = int_{-alpha}^{alpha} p
* quantization density, non-uniform grid (Sec. IV-B, first boxed equation):
      lambda_s(g) = s p(g)^(1/3) / int_{-alpha}^{alpha} p^(1/3)
* truncation threshold, non-uniform grid (Sec. IV-B, second boxed equation):
      same form with Q_N(alpha) = [int_{-alpha}^{alpha} p^(1/3) (1/(2 alpha))^(2/3)]^3
* uniform codebook (Sec. IV-A):  l_k = -alpha + k * 2 alpha / s
* truncated BiScaled quantizer (appendix "Truncated BiScaled Quantization"): two uniform
  regions, s_beta cells on [-beta, beta] and s_alpha on the rest of [-alpha, alpha],
      Q_B(alpha, k) = [(2 int_{k alpha}^{alpha} p)^(1/3) (1-k)^(2/3) + (2 int_0^{k alpha} p)^(1/3) k^(2/3)]^3,
      k* = argmin_k Q_B(alpha, k),  alpha from the boxed equation with Q_B(alpha, k*),
      s_beta / s = p1^(1/3) k / (p2^(1/3) (1-k) + p1^(1/3) k),  s_alpha = s - s_beta,
  p1, p2 the average densities on [0, beta] and [beta, alpha], k = beta / alpha

Readings where the paper is silent (each also listed in the design document):

* p(g) inside [-alpha, alpha] is the empirical, symmetric density given by the
  histogram of |g| (piecewise constant per bin); the power law is used only
  where the paper uses it (the tail term of the alpha equation, gamma, rho).
* g_min, when the caller gives none, is the lower edge of the histogram bin
  holding the 0.9-quantile of |g|; gamma then comes from the binned data, each
  bin standing at the geometric mean of its edges.
* "alternating iterations": start from the Q = 1 value (alpha' of Sec. IV-A),
  iterate the boxed map at most 100 times, stop at relative change 1e-10.
* outside the paper's domain 3 < gamma <= 5 the formulas are applied as
  written for gamma > 2.02 (smaller estimates are lifted to 2.02); an iterate
  beyond max|g| is clamped there ("no truncation"), below g_min to g_min.
* density -> codebook: level l_k is where the integral of lambda_s from -alpha
  reaches k (so that int lambda_s = s, Sec. III-A), mirrored about zero.

Parity unpinned by the paper: the iteration count and tolerance, the choice of
g_min and the candidate set of the BiScaled search are readings; the tests pin
the fixed points and minima they lead to (closed forms, brute force), not the
number of steps taken.
* BiScaled: k is searched over k = 0 and the histogram's bin edges below alpha
  (beta = k alpha is then an edge), the smallest k winning a tie; the boxed
  equation is iterated like the other two with Q = min_k Q_B(alpha, k), k* re-chosen
  at every iterate; s_beta is the odd integer nearest to its real-valued formula,
  within [1, s - 2] (s is odd, so an odd inner count leaves the two outer regions
  the same even share); k* = 0 means a uniform codebook.
"""
import numpy as np

from .binding import GRID_BISCALED, GRID_NONUNIFORM, GRID_UNIFORM, NBINS, PARAMS_DTYPE

FLAG_ALPHA_CLAMPED_MAX = 1    # fixed point at or beyond max|g|: alpha = max|g|
FLAG_GAMMA_CLAMPED = 2        # tail-index estimate below 2.02, lifted
FLAG_NOT_CONVERGED = 4        # 100 iterations without meeting the tolerance
FLAG_DEGENERATE = 8           # no finite non-zero data or no usable tail
FLAG_ALPHA_OVERRIDE = 16      # alpha supplied by the caller (or max|g| asked for)
FLAG_ALPHA_CLAMPED_MIN = 32   # fixed point at or below g_min, lifted

GAMMA_FLOOR = 2.02
ALPHA_FLOOR = 2.0 ** -64
TAIL_QUANTILE_NUM, TAIL_QUANTILE_DEN = 9, 10
MAX_ITER = 100
REL_TOL = 1e-10


def bin_edges(absmax):
    """Lower and upper edge of every histogram bin, as fp64 (all exact)."""
    lo = np.zeros(NBINS)
    hi = np.zeros(NBINS)
    hi[0] = 2.0 ** -40
    for i in range(1, NBINS - 1):
        octave, m = divmod(i - 1, 16)
        lo[i] = (1.0 + m / 16.0) * 2.0 ** (octave - 40)
        hi[i] = (1.0 + (m + 1) / 16.0) * 2.0 ** (octave - 40)
    lo[NBINS - 1] = 2.0 ** 16
    hi[NBINS - 1] = max(float(absmax), 2.0 ** 17)
    return lo, hi


class Density:
    """Empirical symmetric density of g from the histogram of |g|."""

    def __init__(self, hist, absmax):
        self.hist = np.asarray(hist, dtype=np.float64)
        self.n = float(self.hist.sum())
        self.absmax = float(absmax)
        self.lo, self.hi = bin_edges(absmax)
        self.w = self.hi - self.lo
        # two-sided density on the bin: half the bin's mass on each side of 0
        self.p = self.hist / (2.0 * self.n * self.w) if self.n > 0 else np.zeros(NBINS)
        self.p13 = np.cbrt(self.p)

    def Q_U(self, alpha):
        """int_{-alpha}^{alpha} p: fraction of |g| <= alpha, linear inside a bin."""
        covered = np.clip(alpha - self.lo, 0.0, self.w)
        return float(np.sum(self.hist * (covered / self.w)) / self.n)

    def half_int_p13(self, x):
        """H(x) = int_0^x p^(1/3)."""
        covered = np.clip(x - self.lo, 0.0, self.w)
        return float(np.sum(self.p13 * covered))

    def Q_N(self, alpha):
        return (2.0 * self.half_int_p13(alpha)) ** 3 / (2.0 * alpha) ** 2

    def Q_B(self, alpha, k):
        """Q_B(alpha, k) of the BiScaled appendix, for any 0 <= k <= 1."""
        c_a = self.Q_U(alpha)                       # 2 int_0^alpha p
        c_b = self.Q_U(k * alpha)                   # 2 int_0^{k alpha} p
        outer = max(c_a - c_b, 0.0)
        return (np.cbrt(outer) * (1.0 - k) ** (2.0 / 3.0) + np.cbrt(c_b) * k ** (2.0 / 3.0)) ** 3

    def best_k(self, alpha):
        """(j, Q_B(alpha, lo_j / alpha)) minimising Q_B over beta in {0} U {bin edges lo_j < alpha};
        j = 0 stands for beta = 0.  The smallest beta wins a tie."""
        best_j, best_q = 0, self.Q_B(alpha, 0.0)
        for j in range(1, NBINS):
            if self.lo[j] >= alpha:
                break
            q = self.Q_B(alpha, self.lo[j] / alpha)
            if q < best_q:
                best_j, best_q = j, q
        return best_j, best_q

    def inv_half_int_p13(self, t):
        """Smallest x >= 0 with H(x) >= t."""
        acc = 0.0
        for i in range(NBINS):
            step = self.p13[i] * self.w[i]
            if step > 0.0 and acc + step >= t:
                return self.lo[i] + (t - acc) / self.p13[i]
            acc += step
        return self.hi[NBINS - 1]


def estimate_tail(stats, dens):
    """(g_min, n_tail, sum_log) -- exact terms if the caller fixed g_min, else binned."""
    if float(stats["g_min"]) > 0.0:
        return float(stats["g_min"]), float(stats["n_tail"]), float(stats["sum_log_tail"])
    cum = 0.0
    j = NBINS - 1
    for i in range(NBINS):
        cum += dens.hist[i]
        if TAIL_QUANTILE_DEN * cum >= TAIL_QUANTILE_NUM * dens.n:
            j = i
            break
    if j == 0:
        return 0.0, 0.0, 0.0
    g_min = dens.lo[j]
    n_tail = 0.0
    sum_log = 0.0
    for i in range(j, NBINS):
        rep = np.sqrt(dens.lo[i] * dens.hi[i]) if i < NBINS - 1 else dens.lo[i]
        n_tail += dens.hist[i]
        sum_log += dens.hist[i] * np.log(rep / g_min)
    return g_min, n_tail, sum_log


def solve_alpha(dens, g_min, gamma, rho, s, grid):
    """Fixed point of the boxed alpha equation (uniform: Q_U, non-uniform: Q_N)."""
    flags = 0
    if grid == GRID_UNIFORM:
        Q = dens.Q_U
    elif grid == GRID_NONUNIFORM:
        Q = dens.Q_N
    else:
        def Q(a):
            return dens.best_k(a)[1]
    a_min = g_min * (1.0 + 2.0 ** -10)
    a_max = dens.absmax
    C = 2.0 * rho * s * s / (gamma - 2.0)

    def clamp(a):
        return min(max(a, a_min), a_max)

    a = clamp(g_min * C ** (1.0 / (gamma - 1.0)))
    converged = False
    for _ in range(MAX_ITER):
        q = Q(a)
        a_new = clamp(g_min * (C / q) ** (1.0 / (gamma - 1.0))) if q > 0.0 else a_max
        if abs(a_new - a) <= REL_TOL * a_new:
            a = a_new
            converged = True
            break
        a = a_new
    if not converged:
        flags |= FLAG_NOT_CONVERGED
    if a >= a_max:
        flags |= FLAG_ALPHA_CLAMPED_MAX
    elif a <= a_min:
        flags |= FLAG_ALPHA_CLAMPED_MIN
    return a, flags


def uniform_levels(alpha_f, s):
    a = float(alpha_f)
    lv = np.array([-a + k * (2.0 * a / s) for k in range(s + 1)]).astype(np.float32)
    lv[s] = np.float32(a)
    return lv


def nonuniform_levels(dens, alpha_f, s):
    a = float(alpha_f)
    half = dens.half_int_p13(a)
    lv = np.zeros(s + 1)
    lv[0], lv[s] = -a, a
    for k in range((s + 1) // 2, s):
        x = min(dens.inv_half_int_p13(half * (2 * k - s) / s), a)
        lv[k], lv[s - k] = x, -x
    return lv.astype(np.float32)


def biscaled_split(dens, alpha_f, s):
    """(beta, s_beta) of the BiScaled codebook at threshold alpha_f; beta = 0: uniform."""
    a = float(alpha_f)
    j, _ = dens.best_k(a)
    if j == 0:
        return 0.0, s
    beta = dens.lo[j]
    k = beta / a
    c_b, c_a = dens.Q_U(beta), dens.Q_U(a)
    p1 = c_b / (2.0 * beta)                         # average density on [0, beta]
    p2 = max(c_a - c_b, 0.0) / (2.0 * (a - beta))   # and on [beta, alpha]
    inner, outer = np.cbrt(p1) * k, np.cbrt(p2) * (1.0 - k)
    x = s * inner / (inner + outer) if inner + outer > 0.0 else float(s)
    s_beta = 2 * int(np.floor((x - 1.0) / 2.0 + 0.5)) + 1      # nearest odd integer
    return beta, min(max(s_beta, 1), s - 2)


def biscaled_levels(dens, alpha_f, s):
    a = float(alpha_f)
    beta, s_beta = biscaled_split(dens, alpha_f, s)
    if beta <= 0.0:
        return uniform_levels(alpha_f, s)
    half_outer = (s - s_beta) // 2                  # cells on each side beyond beta
    lv = np.zeros(s + 1)
    for j in range(s_beta + 1):
        lv[half_outer + j] = -beta + j * (2.0 * beta / s_beta)
    lv[half_outer], lv[half_outer + s_beta] = -beta, beta
    for j in range(1, half_outer + 1):
        x = beta + j * ((a - beta) / half_outer)
        lv[half_outer + s_beta + j], lv[half_outer - j] = x, -x
    lv[0], lv[s] = -a, a
    return lv.astype(np.float32)


def tq_params_one(stats, bits, grid, alpha_override=0.0):
    """One PARAMS_DTYPE record from one STATS_DTYPE record.

    alpha_override > 0: use it; < 0: alpha = max|g| (quantization without
    truncation, the QSGD / NQSGD comparison of Sec. V); 0: the paper's formula.
    """
    s = (1 << bits) - 1
    P = np.zeros((), dtype=PARAMS_DTYPE)
    P["bits"], P["s"], P["grid"] = bits, s, grid
    dens = Density(stats["hist"], stats["absmax"])
    flags = 0
    g_min = gamma = rho = 0.0
    if dens.n <= 0 or dens.absmax <= 0.0:
        flags |= FLAG_DEGENERATE                 # nothing to design from; a given threshold still holds
        alpha = ALPHA_FLOOR
        if alpha_override > 0.0:
            flags |= FLAG_ALPHA_OVERRIDE
            alpha = float(alpha_override)
    else:
        g_min, n_tail, sum_log = estimate_tail(stats, dens)
        tail_ok = g_min > 0.0 and n_tail > 0 and sum_log > 0.0 and g_min < dens.absmax
        if tail_ok:
            gamma = 1.0 + n_tail / sum_log                    # Sec. V, MLE
            rho = n_tail / (2.0 * dens.n)                     # one-sided tail mass
        if alpha_override != 0.0:
            flags |= FLAG_ALPHA_OVERRIDE
            alpha = float(alpha_override) if alpha_override > 0.0 else dens.absmax
        elif not tail_ok:
            flags |= FLAG_DEGENERATE
            alpha = dens.absmax
        else:
            g_used = gamma
            if g_used < GAMMA_FLOOR:
                g_used = GAMMA_FLOOR
                flags |= FLAG_GAMMA_CLAMPED
            alpha, f = solve_alpha(dens, g_min, g_used, rho, s, grid)
            flags |= f
    alpha_f = np.float32(max(alpha, ALPHA_FLOOR))
    if grid == GRID_UNIFORM or dens.half_int_p13(float(alpha_f)) <= 0.0:
        lv = uniform_levels(alpha_f, s)      # (no mass inside [-alpha, alpha]: nothing to shape)
    elif grid == GRID_NONUNIFORM:
        lv = nonuniform_levels(dens, alpha_f, s)
    else:
        lv = biscaled_levels(dens, alpha_f, s)
    inv_w = np.zeros(16, dtype=np.float32)
    if grid == GRID_UNIFORM:
        inv_w[:s] = np.float32(s / (2.0 * float(alpha_f)))
    else:
        for k in range(s):
            width = float(lv[k + 1]) - float(lv[k])
            if width > 0.0:
                iw = np.float64(1.0 / width)
                inv_w[k] = np.float32(iw) if iw <= 3.4028234663852886e38 else 0.0
    P["alpha"] = alpha_f
    P["level"][: s + 1] = lv
    P["inv_w"] = inv_w
    P["gamma_hat"], P["rho_hat"], P["g_min"] = gamma, rho, g_min
    P["flags"] = flags
    return P


def tq_params(stats, bits, grid, alpha_override=0.0):
    """One record per bucket."""
    stats = np.atleast_1d(stats)
    out = np.zeros(stats.size, dtype=PARAMS_DTYPE)
    for b in range(stats.size):
        out[b] = tq_params_one(stats[b], bits, grid, alpha_override)
    return out
