"""Pins for the oracle's fused server step (Alg. 1: aggregate, then theta <- theta - eta g_bar;
momentum and weight decay as in the experiments of Sec. V): exact dyadic known answers,
closed forms of the momentum recursion, and special cases that reduce to the plain
aggregate."""
import numpy as np
import pytest

from oracle import binding as O
from test_oracle_quantizer import make_params, uniform_params

DYADIC = [-1.0, -0.5, 0.5, 1.0]           # a 2-bit codebook whose sums and halves are exact


def on_grid_payload(values, P, worker):
    """Values lying on levels encode without randomness (a pinned property of the quantizer)."""
    return O.compress(np.asarray(values, dtype=np.float32), P, 3, worker, 0)


def two_workers(v0, v1):
    P = make_params(DYADIC, O.GRID_NONUNIFORM)
    return [on_grid_payload(v0, P, 0), on_grid_payload(v1, P, 1)], [P, P]


def test_plain_sgd_known_answer():
    # g_bar = ((1) + (0.5)) / 2 = 0.75, ((-1) + (-1)) / 2 = -1, ((0.5) + (-0.5)) / 2 = 0
    pays, Ps = two_workers([1.0, -1.0, 0.5], [0.5, -1.0, -0.5])
    theta = np.array([10.0, 10.0, 10.0], dtype=np.float32)
    O.decompress_aggregate_update(pays, Ps, theta, 2, eta=0.5)
    assert theta.tolist() == [10.0 - 0.375, 10.5, 10.0]


def test_momentum_recursion_closed_form():
    # constant g_bar = c: v_t = c (1 - mu^t) / (1 - mu), theta_T = theta_0 - eta sum_t v_t
    pays, Ps = two_workers([1.0] * 4, [0.5] * 4)              # c = 0.75
    theta = np.full(4, 8.0, dtype=np.float32)
    vel = np.zeros(4, dtype=np.float32)
    c, mu, eta, T = 0.75, 0.5, 0.25, 6
    for _ in range(T):
        O.decompress_aggregate_update(pays, Ps, theta, 2, eta=eta, momentum=mu, velocity=vel)
    v_T = c * (1 - mu ** T) / (1 - mu)
    sum_v = sum(c * (1 - mu ** t) / (1 - mu) for t in range(1, T + 1))
    assert vel.tolist() == [v_T] * 4                          # dyadic: exact in binary32
    assert theta.tolist() == [8.0 - eta * sum_v] * 4


def test_weight_decay_alone_shrinks_theta():
    # mirrored workers: g_bar = 0, so theta <- theta - eta (wd theta)
    pays, Ps = two_workers([1.0, 0.5, -0.5], [-1.0, -0.5, 0.5])
    theta = np.array([2.0, -4.0, 0.0], dtype=np.float32)
    O.decompress_aggregate_update(pays, Ps, theta, 2, eta=0.5, weight_decay=0.25)
    assert theta.tolist() == [1.75, -3.5, 0.0]


def test_weight_decay_enters_the_velocity():
    pays, Ps = two_workers([1.0], [1.0])                      # g_bar = 1
    theta = np.array([4.0], dtype=np.float32)
    vel = np.array([2.0], dtype=np.float32)
    O.decompress_aggregate_update(pays, Ps, theta, 2, eta=0.125, momentum=0.5, weight_decay=0.25,
                                  velocity=vel)
    assert vel.tolist() == [0.5 * 2.0 + (1.0 + 0.25 * 4.0)]   # 3
    assert theta.tolist() == [4.0 - 0.125 * 3.0]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("be", [0, 256])
def test_reduces_to_the_plain_aggregate(bits, be):
    """eta = -1 on theta = 0 returns g_bar itself; eta = 0 changes nothing but the velocity."""
    d, N = 1000, 3
    rng = np.random.default_rng(bits + be)
    nb = 1 if be == 0 else (d + be - 1) // be
    Ps = [np.concatenate([uniform_params(0.5 + 0.25 * i + 0.1 * b, bits) for b in range(nb)]) for i in range(N)]
    pays = [O.compress(rng.standard_normal(d).astype(np.float32), Ps[i], 7, i, 1, bucket_elems=be) for i in range(N)]
    g_bar = O.decompress_aggregate(pays, Ps, d, bits, bucket_elems=be)
    theta = np.zeros(d, dtype=np.float32)
    O.decompress_aggregate_update(pays, Ps, theta, bits, eta=-1.0, bucket_elems=be)
    assert (theta == g_bar).all()
    theta0 = rng.standard_normal(d).astype(np.float32)
    theta, vel = theta0.copy(), np.zeros(d, dtype=np.float32)
    O.decompress_aggregate_update(pays, Ps, theta, bits, eta=0.0, momentum=0.9, velocity=vel, bucket_elems=be)
    assert (theta == theta0).all() and (vel == g_bar).all()
    # general case against the recursion evaluated by numpy in binary32, one rounding per step
    w = np.array([0.5, 0.25, 0.25], dtype=np.float32)
    g_w = O.decompress_aggregate(pays, Ps, d, bits, bucket_elems=be, weights=w)
    theta, vel = theta0.copy(), g_bar.copy()
    O.decompress_aggregate_update(pays, Ps, theta, bits, eta=0.01, momentum=0.9, weight_decay=5e-4,
                                  velocity=vel, bucket_elems=be, weights=w)
    f = np.float32
    u = g_w + f(5e-4) * theta0
    v = f(0.9) * g_bar + u
    assert (vel == v).all() and (theta == theta0 - f(0.01) * v).all()


def test_momentum_argument_is_ignored_without_a_velocity():
    pays, Ps = two_workers([1.0, -0.5], [0.5, -0.5])
    a = np.array([1.0, 1.0], dtype=np.float32)
    b = a.copy()
    O.decompress_aggregate_update(pays, Ps, a, 2, eta=0.5, momentum=0.9)
    O.decompress_aggregate_update(pays, Ps, b, 2, eta=0.5)
    assert (a == b).all()
