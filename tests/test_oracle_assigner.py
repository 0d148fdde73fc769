"""Pins of the assignment oracle (Sec. 4.2): closed forms, exact enumeration, the separable one-pair case."""
import numpy as np
import pytest

from oracle import assigner as A


def _instance(rng, n, n_peers, spread=4.0):
    beta = np.exp(rng.normal(0.0, spread, size=n)).astype(np.float32)
    peer = np.sort(rng.integers(0, n_peers, size=n)).astype(np.int32)
    theta = rng.uniform(0.2, 3.0, size=n_peers) * 1e-3
    gamma = rng.uniform(0.0, 0.5, size=n_peers)
    return beta, peer, theta, gamma


def test_objective_by_hand():
    # Eq. 8: 9/(2^2-1)^2 + 225/(2^4-1)^2 = 2;  Eq. 7: 0.5 * (10*2 + 10*4) + 1 = 31;  Eq. 9 at lambda 1/4
    f, var, t = A.objective([9.0, 225.0], [0, 0], 1, 10, [2, 4], 0.25, [0.5], [1.0])
    assert var == 2.0 and t == 31.0 and f == 0.25 * 2.0 + 0.75 * 31.0
    # two pairs: the slower one sets the time; a pair without messages is ignored
    f, var, t = A.objective([9.0, 65025.0], [0, 2], 3, 4, [2, 8], 0.5, [1.0, 100.0, 0.25], [0.0, 1e9, 3.0])
    assert var == 2.0 and t == max(1.0 * 8, 0.25 * 32 + 3.0) and f == 0.5 * 2.0 + 0.5 * 11.0


def test_groups_are_runs_of_descending_beta():
    beta = np.array([1.0, 7.0, 3.0, 7.0, 0.5, 2.0, 9.0], dtype=np.float32)
    peer = np.array([0, 0, 0, 0, 0, 1, 1], dtype=np.int32)
    g = A.make_groups(beta, peer, 3, 2)
    assert g == [[[1, 3], [2, 0], [4]], [[6, 5]], []]


@pytest.mark.parametrize("seed", range(12))
def test_one_pair_is_separable_and_greedy_is_exact(seed):
    """With one device pair Eq. 9 splits into one term per group:
    lambda*B_g/(2^b-1)^2 + (1-lambda)*theta*n_g*D*b, plus a constant - so the optimum is a per-group argmin."""
    rng = np.random.default_rng(seed)
    n, gs, dim = int(rng.integers(3, 17)), int(rng.integers(1, 4)), int(rng.integers(1, 40))
    beta, peer, theta, gamma = _instance(rng, n, 1)
    lam = float(rng.uniform(0.05, 0.95))
    groups = A.make_groups(beta, peer, 1, gs)[0]
    want = np.zeros(n, dtype=np.uint8)
    for members in groups:
        B = float(sum(float(beta[k]) for k in members))
        cost = {b: lam * B * A.inv_levels_sq(b) + (1 - lam) * theta[0] * len(members) * dim * b for b in A.WIDTHS}
        want[members] = min(A.WIDTHS, key=lambda b: cost[b])
    f_want, _, _ = A.objective(beta, peer, 1, dim, want, lam, theta, gamma)
    got = A.greedy(beta, peer, 1, dim, gs, lam, theta, gamma)
    f_got, _, _ = A.objective(beta, peer, 1, dim, got, lam, theta, gamma)
    assert f_got == pytest.approx(f_want, rel=1e-12)
    if len(groups) <= 8:
        _, f_best = A.brute_force(beta, peer, 1, dim, gs, lam, theta, gamma)
        assert f_best == pytest.approx(f_want, rel=1e-12)


@pytest.mark.parametrize("seed", range(10))
def test_several_pairs_against_enumeration(seed):
    rng = np.random.default_rng(100 + seed)
    n_peers = int(rng.integers(2, 4))
    n, gs, dim = int(rng.integers(4, 9)), 1, int(rng.integers(1, 20))
    beta, peer, theta, gamma = _instance(rng, n, n_peers, spread=2.0)
    lam = float(rng.uniform(0.05, 0.95))
    got = A.greedy(beta, peer, n_peers, dim, gs, lam, theta, gamma)
    assert set(np.unique(got)) <= {2, 4, 8}
    f_got, _, _ = A.objective(beta, peer, n_peers, dim, got, lam, theta, gamma)
    _, f_best = A.brute_force(beta, peer, n_peers, dim, gs, lam, theta, gamma)
    assert f_got >= f_best * (1 - 1e-12)
    # a pair's prefix misses its best packing by less than one upgrade: the largest single gain, per pair
    slack = 0.0
    for i in range(n_peers):
        b_i = [float(b) for b, q in zip(beta, peer) if q == i]
        if b_i:
            slack += max(b_i) * (A.inv_levels_sq(2) - A.inv_levels_sq(4))
    assert f_got <= f_best + lam * slack * (1 + 1e-12)


def test_extremes_of_lambda():
    rng = np.random.default_rng(7)
    beta, peer, theta, gamma = _instance(rng, 40, 3)
    dim = 16
    assert np.all(A.greedy(beta, peer, 3, dim, 4, 1.0, theta, gamma) == 8)          # variance only
    bits = A.greedy(beta, peer, 3, dim, 4, 0.0, theta, gamma)                        # time only
    _, _, t = A.objective(beta, peer, 3, dim, bits, 0.0, theta, gamma)
    t_all2 = max(theta[i] * dim * 2 * np.sum(peer == i) + gamma[i] for i in range(3))
    assert t == pytest.approx(t_all2, rel=1e-15)
    straggler = int(np.argmax([theta[i] * dim * 2 * np.sum(peer == i) + gamma[i] for i in range(3)]))
    assert np.all(bits[peer == straggler] == 2)


def test_widths_follow_beta_within_a_pair():
    rng = np.random.default_rng(11)
    beta, peer, theta, gamma = _instance(rng, 300, 3)
    bits = A.greedy(beta, peer, 3, 64, 10, 0.5, theta * 1e-2, gamma)
    assert len(np.unique(bits)) == 3                       # the instance is not degenerate
    for i in range(3):
        idx = np.nonzero(peer == i)[0]
        full = len(idx) // 10 * 10                         # equal-sized groups only: the ragged one has its own cost
        order = idx[np.lexsort((idx, -beta[idx].astype(np.float64)))][:full]
        assert np.all(np.diff(bits[order].astype(np.int32)) <= 0)
        for s in range(0, full, 10):
            assert len(np.unique(bits[order[s: s + 10]])) == 1
