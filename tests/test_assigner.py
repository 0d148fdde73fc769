"""adaqp_assign_bits (host code of the library) against the assignment oracle: identical widths, and the reported
objective against the oracle's definition of Eq. 9."""
import numpy as np
import pytest

from oracle import assigner as A
from paper_2306_01381_amd import binding as B


def _instance(rng, n, n_peers, spread):
    beta = np.exp(rng.normal(0.0, spread, size=n)).astype(np.float32)
    beta[rng.random(n) < 0.05] = 0.0                              # constant rows have no quantisation error
    if n > 10:
        beta[3] = beta[7]                                         # a tie
    peer = np.sort(rng.integers(0, n_peers, size=n)).astype(np.int32)
    theta = rng.uniform(0.2, 3.0, size=n_peers) * 10.0 ** rng.uniform(-6, -2)
    gamma = rng.uniform(0.0, 0.5, size=n_peers)
    return beta, peer, theta, gamma


@pytest.mark.parametrize("seed", range(25))
def test_widths_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    n_peers = int(rng.integers(1, 8))
    n = int(rng.integers(1, 400))
    dim = int(rng.choice([1, 7, 128, 602]))
    gs = int(rng.choice([1, 3, 10, 50, 1000]))
    lam = float(rng.choice([0.0, 1.0, rng.uniform(0, 1), 0.5]))
    beta, peer, theta, gamma = _instance(rng, n, n_peers, float(rng.uniform(0.5, 5)))
    want = A.greedy(beta, peer, n_peers, dim, gs, lam, theta, gamma)
    got, obj = B.adaqp_assign_bits(beta, peer, n_peers, dim, gs, lam, theta, gamma)
    assert np.array_equal(got, want)
    f, var, t = A.objective(beta, peer, n_peers, dim, got, lam, theta, gamma)
    assert obj[1] == pytest.approx(var, rel=1e-12) and obj[2] == pytest.approx(t, rel=1e-12)
    assert obj[0] == pytest.approx(f, rel=1e-12)


def test_unsorted_peers_and_a_pair_without_messages():
    rng = np.random.default_rng(99)
    beta, peer, theta, gamma = _instance(rng, 200, 5, 3.0)
    peer = rng.permutation(peer)
    peer[peer == 2] = 4                                           # pair 2 exchanges nothing
    gamma[2] = 1e9                                                # ... so its constant must not set the time
    want = A.greedy(beta, peer, 5, 64, 8, 0.3, theta, gamma)
    got, obj = B.adaqp_assign_bits(beta, peer, 5, 64, 8, 0.3, theta, gamma)
    assert np.array_equal(got, want) and obj[2] < 1e8


def test_exact_on_one_pair_against_enumeration():
    rng = np.random.default_rng(5)
    beta, peer, theta, gamma = _instance(rng, 8, 1, 2.0)
    got, obj = B.adaqp_assign_bits(beta, peer, 1, 16, 1, 0.4, theta, gamma)
    _, f_best = A.brute_force(beta, peer, 1, 16, 1, 0.4, theta, gamma)
    assert obj[0] == pytest.approx(f_best, rel=1e-12)


def test_argument_checks():
    ok = dict(beta_host=np.ones(4, np.float32), peer_of_slot_host=np.zeros(4, np.int32), n_peers=2, dim=8,
              group_size=2, lam=0.5, theta=np.ones(2), gamma=np.zeros(2))
    B.adaqp_assign_bits(**ok)
    bits, obj = B.adaqp_assign_bits(**{**ok, "beta_host": np.zeros(0, np.float32),
                                       "peer_of_slot_host": np.zeros(0, np.int32)})
    assert bits.shape == (0,) and obj.tolist() == [0.0, 0.0, 0.0]
    for bad in ({"lam": 1.5}, {"lam": float("nan")}, {"group_size": 0}, {"dim": 0},
                {"beta_host": np.array([1, -1, 1, 1], np.float32)},
                {"beta_host": np.array([1, np.nan, 1, 1], np.float32)},
                {"beta_host": np.array([1, np.inf, 1, 1], np.float32)},
                {"peer_of_slot_host": np.array([0, 2, 0, 0], np.int32)},
                {"theta": np.array([1.0, -1.0])}):
        with pytest.raises(B.AdaqpError):
            B.adaqp_assign_bits(**{**ok, **bad})
