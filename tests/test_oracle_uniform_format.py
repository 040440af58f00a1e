"""The uniform codebook's wire-format rule against Eq. (2) taken step by step.

On every codebook the oracle's code is Eq. (2) as written: the cell by comparison with the
levels, p_r = (g - l_k)/|Delta_k|, the upper end iff a uniform variate is <= p_r
(``tqo_quantize_eq2``).  On the uniform codebook (Sec. IV-A, l_k = -alpha + k 2alpha/s) the
format states the same thing as stochastic rounding of the position, floor(t + U), evaluated
with two fused multiply-adds (``tqo_quantize_one``).  These tests pin the second statement to
the first by enumerating all 65,536 draws: same cell, and the number of upward draws equal
to within ONE draw, for inputs on every level, on its binary32 neighbours, between levels,
at and beyond +-alpha, at zero and at subnormals; and they show that the criterion rejects
the mistakes one could plausibly make in the position form (a dropped half grain, a cell
offset by one, a reciprocal of the wrong width).
"""
import numpy as np
import pytest

from oracle import binding as O
from test_oracle_quantizer import NONUNIFORM_3, NONUNIFORM_7, make_params, uniform_params

ALPHAS = [1.0, 0.3, 3.5, 0.1, 123.456, 7.07e-4, 7.0710678e-4, 1e-30, 2.0 ** -64, 1e30]


def neighbours(x, n):
    """x and its n binary32 neighbours on each side."""
    out = [np.float32(x)]
    for direction in (np.float32(np.inf), np.float32(-np.inf)):
        y = np.float32(x)
        for _ in range(n):
            y = np.nextafter(y, direction, dtype=np.float32)
            out.append(y)
    return out


def probe_values(P, n_random, seed):
    s = int(P["s"][0])
    lv = P["level"][0, : s + 1]
    alpha = float(P["alpha"][0])
    xs = []
    for l in lv:
        xs += neighbours(l, 3)
    xs += [np.float32((float(lv[k]) + float(lv[k + 1])) / 2) for k in range(s)]
    xs += list(np.random.default_rng(seed).uniform(-alpha, alpha, n_random).astype(np.float32))
    xs += [np.float32(v) for v in (0.0, -0.0, 1e-45, -1e-45, 1e-39, -1e-39, 2 * alpha, -2 * alpha,
                                   np.inf, -np.inf, np.nan)]
    return xs, lv


def plain_cell(x, lv, alpha):
    """Index k of the cell [l_k, l_{k+1}] holding T_alpha(x), by bisection in fp64."""
    x = 0.0 if np.isnan(x) else float(x)
    xc = min(max(x, -alpha), alpha)
    k = int(np.searchsorted(lv.astype(np.float64), xc, side="right")) - 1
    return min(max(k, 0), lv.size - 2)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_position_form_agrees_with_eq2_within_one_draw(bits):
    worst = 0
    codes = np.arange(16)
    for a_i, alpha in enumerate(ALPHAS):
        P = uniform_params(alpha, bits)
        xs, lv = probe_values(P, 120, seed=bits * 100 + a_i)
        signed = []
        for x in xs:
            fmt = O.enumerate_draws(x, P, eq2=False).astype(np.int64)
            eq2 = O.enumerate_draws(x, P, eq2=True).astype(np.int64)
            k = plain_cell(x, lv, float(P["alpha"][0]))
            # both statements stay inside the cell Eq. (2) names ...
            outside = [c for c in range(16) if c not in (k, k + 1)]
            assert eq2[outside].sum() == 0 and fmt[outside].sum() == 0, (alpha, float(x), fmt, eq2)
            # ... and send the same number of draws upward, to within one
            diff = int(np.abs(fmt - eq2).max())
            worst = max(worst, diff)
            assert diff <= 1, (alpha, float(x), fmt[: lv.size], eq2[: lv.size])
            signed.append(int(((fmt - eq2) * codes).sum()))
        # ... with no systematic direction: the single draw goes either way
        assert abs(np.mean(signed)) < 0.1, (alpha, np.mean(signed))
    assert worst <= 1


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_a_larger_draw_never_lowers_the_code_in_either_statement(bits):
    """Both statements use the draw in the same direction, so 'same counts' means the same
    decision for every draw but at most one."""
    P = uniform_params(0.3, bits)
    xs, _ = probe_values(P, 10, seed=1)
    for x in xs[::5]:
        for fn in (O.quantize_one, O.quantize_eq2):
            c = np.array([fn(x, P, r) for r in range(0, 65536, 251)] + [fn(x, P, 65535)])
            assert (np.diff(c) >= 0).all()


def position_form_counts(x, alpha, inv_w, s, offset, grain):
    """numpy restatement of floor(fma(r, 2^-16, fma(xc, inv_w, offset))) over all draws, with
    the constants left open so that wrong ones can be planted.  fp64 holds both fused
    multiply-adds of binary32 operands exactly before the single rounding."""
    x = np.float32(0.0) if np.isnan(x) else np.float32(x)
    xc = np.float32(min(max(x, np.float32(-alpha)), np.float32(alpha)))
    u = np.float32(np.float64(xc) * np.float64(inv_w) + np.float64(np.float32(offset)))
    r = np.arange(65536, dtype=np.float64)
    v = (r * np.float64(grain) + np.float64(u)).astype(np.float32)
    code = np.clip(np.floor(v).astype(np.int64), 0, s)
    return np.bincount(code, minlength=16)


def test_the_criterion_rejects_planted_mistakes():
    bits, alpha = 3, np.float32(0.3)
    P = uniform_params(alpha, bits)
    s = 7
    inv_w = P["inv_w"][0, 0]
    xs, lv = probe_values(P, 60, seed=3)
    xs = [x for x in xs if np.isfinite(x)]

    codes = np.arange(16)

    def verdict(offset, grain, iw=inv_w):
        """(largest difference of a code's count, some draw leaves Eq. (2)'s cell, mean signed
        difference of the number of upward draws) of the position form with these constants."""
        w, leaves, signed = 0, False, []
        for x in xs:
            eq2 = O.enumerate_draws(x, P, eq2=True).astype(np.int64)
            got = position_form_counts(x, alpha, iw, s, offset, grain)
            w = max(w, int(np.abs(got - eq2).max()))
            leaves = leaves or bool(got[eq2 == 0].sum())
            signed.append(int(((got - eq2) * codes).sum()))
        return w, leaves, float(np.mean(signed))

    def accepted(v):
        return v[0] <= 1 and not v[1] and abs(v[2]) < 0.1

    good_offset = 0.5 * s + 2.0 ** -17
    # the restatement with the format's constants reproduces the oracle's counts exactly ...
    for x in xs:
        assert (position_form_counts(x, alpha, inv_w, s, good_offset, 2.0 ** -16)
                == O.enumerate_draws(x, P, eq2=False)).all()
    # ... and is accepted; each planted mistake is rejected
    assert accepted(verdict(good_offset, 2.0 ** -16))
    dropped = verdict(0.5 * s, 2.0 ** -16)                       # half grain dropped: p_r rounded down, not to
    assert dropped[1] and dropped[2] < -0.3 and not accepted(dropped)  # nearest; a level is not always kept
    assert not accepted(verdict(0.5 * s + 2.0 ** -16, 2.0 ** -16))         # a whole grain instead of half
    assert not accepted(verdict(0.5 * s + 1.0 + 2.0 ** -17, 2.0 ** -16))   # cell offset by one
    assert not accepted(verdict(0.5 * (s + 1) + 2.0 ** -17, 2.0 ** -16))   # s + 1 levels mistaken for s cells
    assert not accepted(verdict(good_offset, 2.0 ** -15))                  # draw scaled as 15 bits
    assert not accepted(verdict(good_offset, 2.0 ** -16, np.float32((s + 1) / (2 * float(alpha)))))  # wrong width


@pytest.mark.parametrize("P", [uniform_params(1.0, 2), uniform_params(7.07e-4, 3), uniform_params(0.3, 4),
                               make_params(NONUNIFORM_7, O.GRID_NONUNIFORM),
                               make_params(NONUNIFORM_3, O.GRID_NONUNIFORM),
                               make_params([-0.05, -0.01, 0.02, 0.05], O.GRID_NONUNIFORM)])
def test_lemma1_at_and_next_to_every_level(P):
    """Lemma 1 (unbiased; variance (g - l_k)(l_{k+1} - g)) by enumeration of every draw, for the
    wire format's code, on the inputs where the cell decision is delicate: every level, its
    neighbours in binary32, +-alpha, zero, subnormals, mid-cells."""
    s = int(P["s"][0])
    xs, lv32 = probe_values(P, 40, seed=11)
    lv = lv32.astype(np.float64)
    alpha = float(P["alpha"][0])
    for x in xs:
        cnt = O.enumerate_draws(x, P, eq2=False).astype(np.float64)
        xv = 0.0 if np.isnan(x) else float(x)
        xc = min(max(xv, -alpha), alpha)
        k = plain_cell(x, lv32, alpha)
        assert cnt[k] + cnt[k + 1] == 65536
        width = lv[k + 1] - lv[k]
        mean = (cnt[: s + 1] * lv).sum() / 65536
        assert abs(mean - xc) <= width * 2.0 ** -16 + 2e-7 * abs(xc)
        var = (cnt[: s + 1] * (lv - xc) ** 2).sum() / 65536
        assert abs(var - (xc - lv[k]) * (lv[k + 1] - xc)) <= width ** 2 * 2.0 ** -15 + 1e-6 * width * abs(xc)
        assert var <= width ** 2 / 4 * (1 + 1e-6)
