"""tq_decompress_aggregate_update (Alg. 1: aggregate, then theta <- theta - eta g_bar, with
the momentum and weight decay of the Sec. V experiments) against the oracle, bit for bit:
both sides round every product and sum once to binary32 in the same order."""
import numpy as np
import pytest
import torch

from oracle import binding as O
from oracle import params as OP
from paper_2402_01798_amd import binding as B
from paper_2402_01798_amd import synth

pytestmark = pytest.mark.gpu


def make_case(d, N, bits, grid, be, seed):
    """N workers' payloads and parameter records made by the oracle, on host and device."""
    wl = synth.WORKLOADS["cfg4" if be else "cfg2"]
    pays, Ps = [], []
    for i in range(N):
        g = synth.as_numpy(synth.make_gradient(wl, i, "cpu", d))
        P = OP.tq_params(O.stats(g, bucket_elems=be), bits, grid)
        pays.append(O.compress(g, P, seed, i, 2, bucket_elems=be))
        Ps.append(P)
    pays_dev = [torch.from_numpy(p).cuda() for p in pays]
    Ps_dev = [B.params_from_numpy(P) for P in Ps]
    return pays, Ps, pays_dev, Ps_dev


@pytest.mark.parametrize("N", [1, 3, 8, 16, 21])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("be", [0, 4096 + 128])
def test_update_matches_oracle(N, bits, be):
    d = 3 * 4096 + 2048 + 37                                 # several tiles, a short bucket, a ragged end
    grid = (N + bits) & 1
    pays, Ps, pays_dev, Ps_dev = make_case(d, N, bits, grid, be, seed=N * 10 + bits)
    rng = np.random.default_rng(N + bits)
    theta0 = rng.standard_normal(d).astype(np.float32)
    vel0 = (0.01 * rng.standard_normal(d)).astype(np.float32)
    weights = None if N % 2 else (rng.random(N) / N).astype(np.float32)
    for momentum, wd, with_velocity in [(0.0, 0.0, False), (0.9, 5e-4, True), (0.5, 0.0, True), (0.0, 1e-2, False)]:
        want_t, want_v = theta0.copy(), vel0.copy()
        O.decompress_aggregate_update(pays, Ps, want_t, bits, eta=0.01, momentum=momentum, weight_decay=wd,
                                      velocity=want_v if with_velocity else None, bucket_elems=be,
                                      weights=weights)
        theta = torch.from_numpy(theta0).cuda()
        vel = torch.from_numpy(vel0).cuda()
        B.tq_decompress_aggregate_update(pays_dev, Ps_dev, theta, bits, 0.01, momentum, wd,
                                         vel if with_velocity else None, be, weights)
        torch.cuda.synchronize()
        got_t, got_v = theta.cpu().numpy(), vel.cpu().numpy()
        assert (got_t == want_t).all(), (momentum, wd, with_velocity)
        assert (got_v == want_v).all()                       # untouched when no velocity is passed


def test_two_steps_of_momentum_sgd_follow_the_oracle_and_the_unfused_path():
    d, N, bits = 100_003, 4, 3
    pays, Ps, pays_dev, Ps_dev = make_case(d, N, bits, 0, 0, seed=5)
    theta = torch.zeros(d, dtype=torch.float32, device="cuda")
    vel = torch.zeros(d, dtype=torch.float32, device="cuda")
    want_t, want_v = np.zeros(d, np.float32), np.zeros(d, np.float32)
    for _ in range(2):
        B.tq_decompress_aggregate_update(pays_dev, Ps_dev, theta, bits, 0.1, 0.9, 0.0, vel)
        O.decompress_aggregate_update(pays, Ps, want_t, bits, eta=0.1, momentum=0.9, velocity=want_v)
    torch.cuda.synchronize()
    assert (theta.cpu().numpy() == want_t).all() and (vel.cpu().numpy() == want_v).all()
    # the unfused route: g_bar from tq_decompress_aggregate, the recursion by hand in binary32
    g_bar = torch.empty(d, dtype=torch.float32, device="cuda")
    B.tq_decompress_aggregate(pays_dev, Ps_dev, g_bar, bits)
    g = g_bar.cpu().numpy()
    f = np.float32
    v1 = g
    t1 = -(f(0.1) * v1)
    v2 = f(0.9) * v1 + g
    t2 = t1 - f(0.1) * v2
    assert (want_v == v2).all() and (want_t == t2).all()
