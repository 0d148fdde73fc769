"""Pins for the oracle's random source and buffer layout."""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers(oracle):
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        w = [int(t, 16) for t in line.split()]
        assert len(w) == 10
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in out] == w[6:10]
        n += 1
    assert n == 3


def test_rand16_slices_cover_the_block(oracle):
    seed, slot = 0x0123456789ABCDEF, 0x1_0000_0007
    for block in (0, 5, 75):
        words = oracle.philox4x32_10([block, slot & 0xFFFFFFFF, slot >> 32, 0x41645150],
                                     [seed & 0xFFFFFFFF, seed >> 32])
        expect = []
        for w in words:
            expect += [int(w) & 0xFFFF, int(w) >> 16]
        got = [oracle.rand16(seed, slot, 8 * block + k) for k in range(8)]
        assert got == expect


def test_rand16_depends_on_seed_slot_column(oracle):
    base = [oracle.rand16(1, 2, c) for c in range(64)]
    assert base != [oracle.rand16(2, 2, c) for c in range(64)]
    assert base != [oracle.rand16(1, 3, c) for c in range(64)]
    assert base != [oracle.rand16(1, 2 + 2**32, c) for c in range(64)]
    assert base != [oracle.rand16(1 + 2**32, 2, c) for c in range(64)]
    assert len(set(base)) > 56


def test_rand16_is_uniform(oracle):
    # chi-square over 256 bins of the top byte and of the bottom byte, 2^18 draws
    n = 1 << 18
    draws = np.array([oracle.rand16(42, s, c) for s in range(n // 64) for c in range(64)], dtype=np.int64)
    for sel in (draws >> 8, draws & 0xFF):
        cnt = np.bincount(sel, minlength=256)
        chi2 = ((cnt - n / 256) ** 2 / (n / 256)).sum()
        assert chi2 < 255 + 6 * np.sqrt(2 * 255)       # mean 255, sd sqrt(510); 6 sd
    # neighbouring columns are uncorrelated
    a, b = draws[0::2].astype(np.float64), draws[1::2].astype(np.float64)
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.01


def test_layout_grouping_and_offsets(oracle):
    rng = np.random.default_rng(0)
    for dim in (1, 7, 128, 300, 602):
        n, n_peers = 200, 4
        peer = np.sort(rng.integers(0, n_peers, size=n)).astype(np.int32)
        bits = rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=n)
        perm, off, pbp = oracle.plan_layout(dim, bits, peer, n_peers)
        assert sorted(perm.tolist()) == list(range(n))
        sp, sb = peer[perm], bits[perm].astype(np.int64)
        # (peer, width, original position) is non-decreasing lexicographically
        key = list(zip(sp.tolist(), sb.tolist(), perm.tolist()))
        assert key == sorted(key)
        stride = 4 * -(-dim * sb // 32)
        assert off[0] == 0
        assert np.array_equal(off[1:], np.cumsum(stride)[:-1])          # contiguous, no gaps
        assert pbp[-1] == stride.sum()
        for p in range(n_peers):
            assert pbp[p] == stride[sp < p].sum()
        assert np.all(off % 4 == 0)


def test_layout_empty_peer_and_empty_list(oracle):
    perm, off, pbp = oracle.plan_layout(16, np.array([4, 2], np.uint8), np.array([0, 2], np.int32), 3)
    assert perm.tolist() == [0, 1] and off.tolist() == [0, 8] and pbp.tolist() == [0, 8, 8, 12]
    perm, off, pbp = oracle.plan_layout(16, np.zeros(0, np.uint8), np.zeros(0, np.int32), 2)
    assert perm.size == 0 and pbp.tolist() == [0, 0, 0]


def test_layout_rejects_bad_input(oracle):
    with pytest.raises(ValueError):
        oracle.plan_layout(8, np.array([3], np.uint8), np.array([0], np.int32), 1)
    with pytest.raises(ValueError):
        oracle.plan_layout(8, np.array([2, 2], np.uint8), np.array([1, 0], np.int32), 2)
    with pytest.raises(ValueError):
        oracle.plan_layout(8, np.array([2], np.uint8), np.array([1], np.int32), 1)
