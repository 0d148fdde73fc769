"""CPU oracle of the bit-width assignment problem of Sec. 4.2 (Eq. 7, Eq. 8, Eq. 9).

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing else).  Plain Python loops in IEEE double.

Three things live here:
  * objective()    - the definition: Eq. 9's weighted sum of Eq. 8's variance and the largest pair time of Eq. 7,
                     evaluated for a given per-message assignment;
  * brute_force()  - the exact optimum of Eq. 9 over group-wise assignments, by enumerating all 3^groups
                     (tiny inputs only).  The paper hands the same problem to a MILP solver;
  * greedy()       - the solver-free stand-in, in plain steps: start every group at 2 bits, order each pair's
                     upgrades (2->4, 4->8) by variance removed per transferred bit, and for every pair time that
                     such a prefix can reach, let every pair take the longest prefix that fits under it; keep
                     the best objective.  For one device pair this is exact (the objective is then separable);
                     for several it is within the sum over pairs of one upgrade's gain of the optimum.

Grouping (Sec. 4.2, last paragraph): per device pair, messages in descending beta (ties: ascending slot), cut into
runs of group_size; the last run may be shorter.  All messages of a group share one width.
"""
from __future__ import annotations

import itertools
from typing import List, Sequence, Tuple

import numpy as np

WIDTHS = (2, 4, 8)


def inv_levels_sq(b: int) -> float:
    """1 / (2^b - 1)^2, the factor of beta in Eq. 8."""
    return 1.0 / float((2 ** b - 1) ** 2)


def objective(beta, peer, n_peers: int, dim: int, bits, lam: float, theta, gamma) -> Tuple[float, float, float]:
    """(Eq. 9 value, Eq. 8 variance, largest pair time of Eq. 7) of a per-message assignment."""
    var = 0.0
    for k in range(len(beta)):
        var += float(beta[k]) * inv_levels_sq(int(bits[k]))
    worst = None
    for i in range(n_peers):
        payload = 0
        count = 0
        for k in range(len(beta)):
            if int(peer[k]) == i:
                payload += dim * int(bits[k])
                count += 1
        if count == 0:
            continue                                    # a pair that exchanges nothing takes no time
        t = float(theta[i]) * float(payload) + float(gamma[i])
        worst = t if worst is None or t > worst else worst
    worst = 0.0 if worst is None else worst
    return lam * var + (1.0 - lam) * worst, var, worst


def make_groups(beta, peer, n_peers: int, group_size: int) -> List[List[List[int]]]:
    """groups[i] = list of groups of pair i, each a list of slot numbers."""
    out = []
    for i in range(n_peers):
        members = [k for k in range(len(beta)) if int(peer[k]) == i]
        members.sort(key=lambda k: (-float(beta[k]), k))
        out.append([members[s: s + group_size] for s in range(0, len(members), group_size)])
    return out


def _expand(groups, widths_per_group, n) -> np.ndarray:
    bits = np.zeros(n, dtype=np.uint8)
    it = iter(widths_per_group)
    for pair in groups:
        for g in pair:
            b = next(it)
            for k in g:
                bits[k] = b
    return bits


def brute_force(beta, peer, n_peers: int, dim: int, group_size: int, lam: float, theta, gamma):
    """Exact optimum of Eq. 9 over group-wise assignments.  Returns (bits, objective value)."""
    groups = make_groups(beta, peer, n_peers, group_size)
    n_groups = sum(len(p) for p in groups)
    assert n_groups <= 12, "enumeration is for tiny inputs"
    best_bits, best = None, None
    for choice in itertools.product(WIDTHS, repeat=n_groups):
        bits = _expand(groups, choice, len(beta))
        f, _, _ = objective(beta, peer, n_peers, dim, bits, lam, theta, gamma)
        if best is None or f < best:
            best, best_bits = f, bits
    if best_bits is None:
        best_bits, best = np.zeros(len(beta), dtype=np.uint8), 0.0
    return best_bits, best


def greedy(beta, peer, n_peers: int, dim: int, group_size: int, lam: float, theta, gamma) -> np.ndarray:
    """The stand-in for the solver.  Every sum below runs in the stated order in double precision, and the
    comparisons are the ones written, so that an independent implementation of the same steps lands on the
    same assignment."""
    n = len(beta)
    groups = make_groups(beta, peer, n_peers, group_size)
    w2, w4, w8 = inv_levels_sq(2), inv_levels_sq(4), inv_levels_sq(8)
    paths = []                                          # per pair with messages: (i, items, T[m], V[m])
    for i in range(n_peers):
        if not groups[i]:
            continue
        items = []                                      # (efficiency, group, step, gain, cost)
        v0 = 0.0
        count = 0
        for g, members in enumerate(groups[i]):
            b_g = 0.0
            for k in members:
                b_g += float(beta[k])
            v0 += b_g * w2
            count += len(members)
            for step, (gain_w, add_bits) in enumerate(((w2 - w4, 2), (w4 - w8, 4))):
                gain = b_g * gain_w
                cost = add_bits * len(members) * dim
                items.append((gain / float(cost), g, step, gain, cost))
        items.sort(key=lambda it: (-it[0], it[1], it[2]))
        base = 2 * dim * count
        T = [float(theta[i]) * float(base) + float(gamma[i])]
        V = [v0]
        cost_cum, gain_cum = 0, 0.0
        for (_, _, _, gain, cost) in items:
            cost_cum += cost
            gain_cum += gain
            T.append(float(theta[i]) * float(base + cost_cum) + float(gamma[i]))
            V.append(v0 - gain_cum)
        paths.append((i, items, T, V))
    bits = np.zeros(n, dtype=np.uint8)
    if not paths:
        return bits
    z_min = max(T[0] for (_, _, T, _) in paths)
    candidates = sorted({t for (_, _, T, _) in paths for t in T if t >= z_min})
    best, best_m = None, None
    for z in candidates:
        ms = []
        var, worst = 0.0, None
        for (_, _, T, V) in paths:
            m = 0
            while m + 1 < len(T) and T[m + 1] <= z:
                m += 1
            ms.append(m)
            var += V[m]
            worst = T[m] if worst is None or T[m] > worst else worst
        f = lam * var + (1.0 - lam) * worst
        if best is None or f < best:
            best, best_m = f, ms
    for (i, items, _, _), m in zip(paths, best_m):
        width = [2] * len(groups[i])
        for (_, g, step, _, _) in items[:m]:
            width[g] += 2 if step == 0 else 4
        for g, members in enumerate(groups[i]):
            for k in members:
                bits[k] = width[g]
    return bits
