"""Seeded synthetic graph partitions shaped like the paper's workloads.

This module only *draws inputs*: a CSR partition graph (local rows, local + halo columns, central rows
first), a feature matrix, the per-peer send lists and the per-slot bit-widths.  It contains none of the
method's arithmetic (no quantisation, no packing, no layout sizing, no aggregation); both the CPU oracle
and the HIP path consume the arrays it returns.

The shapes follow the paper's datasets (Table 3: node / edge counts and feature widths), its remote-
neighbour ratios (Table 1: 31-63 % of a marginal node's neighbours are remote) and its remark that traffic
between device pairs is unbalanced (Sec. 2.2, Fig. 2).  No dataset item is reproduced: every array is drawn
from numpy's PCG64 with a fixed seed.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np

__all__ = ["PartitionConfig", "Partition", "CONFIGS", "make_partition", "config_by_name", "alpha_sq_stand_in"]


@dataclass(frozen=True)
class PartitionConfig:
    name: str
    n_local: int
    n_halo: int
    mean_degree: float          # target mean number of neighbours per local row (self-loop excluded)
    dim: int
    n_send: int
    n_peers: int
    feat: str                   # "normal" | "relu" | "heavy_tail" | "grad"
    bits: str                   # "uniform" | "mix_c1" | "all2" | "adaptive"
    backward: bool = False      # True: the CSR handed out is the transposed graph (gradient aggregation)
    seed: int = 0
    draw_inflation: float = 1.0  # extra draws to make up for duplicates removed per row
    stands_in_for: str = ""
    aggregator: str = "gcn"     # coefficients: "gcn" symmetric normalisation | "mean" (GraphSAGE-style, 1 / row degree)
    degree_law: str = "zipf"    # row degrees: "zipf" (Zipf(1.5), clipped) | "lognormal" (sigma 1: a milder skew)


# Zipf(1.5) samples are clipped at this raw value; with the clipped mean (about 170) the largest degree
# lands at roughly 75x the mean degree.
_ZIPF_CLIP = 13000
_POPULARITY_EXPONENT = 0.6


CONFIGS: Dict[str, PartitionConfig] = {
    "c0": PartitionConfig("c0", 2_000, 600, 10, 128, 400, 3, "normal", "uniform", seed=0,
                          stands_in_for="tiny parity partition"),
    "c1": PartitionConfig("c1", 58_000, 40_000, 790, 602, 30_000, 3, "normal", "mix_c1", seed=1,
                          draw_inflation=1.17,
                          stands_in_for="one of 4 partitions of a 233K-node / 114M-edge graph, 602 features"),
    # c1 with a milder degree law (same sizes, same mean degree): not one of the metric's workloads; it checks that the
    # rules that pick the aggregation kernels (tiles, panels) do not hinge on c1's heavy tail
    "c1m": PartitionConfig("c1m", 58_000, 40_000, 425, 602, 30_000, 3, "normal", "mix_c1", seed=1,
                           draw_inflation=1.17, degree_law="lognormal",
                           stands_in_for="c1's sizes with log-normal row degrees (sigma 1) instead of Zipf(1.5)"),
    "c2": PartitionConfig("c2", 306_000, 150_000, 23.4, 256, 120_000, 7, "relu", "all2", seed=2,
                          draw_inflation=1.005,
                          stands_in_for="one of 8 partitions of a 2.45M-node / 62M-edge graph, hidden 256"),
    "c3": PartitionConfig("c3", 179_000, 90_000, 8.9, 300, 80_000, 3, "heavy_tail", "uniform", seed=3,
                          draw_inflation=1.003,
                          stands_in_for="one of 4 partitions of a 716K-node / 7M-edge graph, 300 features"),
    "c4": PartitionConfig("c4", 196_000, 180_000, 83.2, 256, 150_000, 7, "grad", "adaptive",
                          backward=True, seed=4, draw_inflation=1.01,
                          stands_in_for="backward pass, one of 8 partitions of a 1.57M-node / 132M-edge graph"),
}


def config_by_name(name: str) -> PartitionConfig:
    return CONFIGS[name.lower()]


@dataclass
class Partition:
    cfg: PartitionConfig
    # aggregation graph handed to the SpMM (forward: A, rows = local nodes; backward: A^T, rows = all nodes)
    rowptr: np.ndarray          # int64 [n_rows + 1]
    col: np.ndarray             # int32 [nnz], ascending inside a row
    val: np.ndarray             # float32 [nnz]
    n_rows: int
    n_cols: int
    # row ranges of the two aggregation launches (first the one that may overlap the message path)
    overlap_rows: tuple         # forward: central rows [0, n_central); backward: local rows [0, n_local)
    dependent_rows: tuple       # forward: marginal rows [n_central, n_local); backward: halo rows
    n_central: int
    # dense operand of the SpMM: forward [n_local + n_halo, dim] (halo rows prefilled), backward dY [n_local, dim]
    feat: np.ndarray
    # message path
    send_idx: np.ndarray        # int32 [n_send]  row of the send matrix for each slot, slots sorted by peer
    peer_of_slot: np.ndarray    # int32 [n_send]  non-decreasing
    bits: np.ndarray            # uint8 [n_send]  in {2, 4, 8}
    halo_idx: np.ndarray        # int32 [n_send]  destination row of each received slot (forward: halo rows, each
                                # once; backward: local marginal rows the received gradients are added to)
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.col.shape[0])


def _degrees(rng: np.random.Generator, n: int, mean: float, cap: int, law: str = "zipf") -> np.ndarray:
    if law == "zipf":
        raw = np.minimum(rng.zipf(1.5, size=n), _ZIPF_CLIP).astype(np.float64)
    elif law == "lognormal":
        raw = rng.lognormal(0.0, 1.0, size=n)
    else:
        raise ValueError(law)
    deg = np.rint(raw * (mean / raw.mean())).astype(np.int64)
    return np.clip(deg, 1, cap)


def _popularity_sampler(rng: np.random.Generator, n: int):
    """Returns draw(u) mapping uniforms to node ids in [0, n) with a power-law popularity."""
    w = (np.arange(1, n + 1, dtype=np.float64)) ** (-_POPULARITY_EXPONENT)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    perm = rng.permutation(n).astype(np.int64)

    def draw(u: np.ndarray) -> np.ndarray:
        return perm[np.minimum(np.searchsorted(cdf, u, side="right"), n - 1)]

    return draw


def _forward_graph(rng: np.random.Generator, cfg: PartitionConfig):
    """Local rows x (local + halo) columns, central rows first, unique ascending columns, self-loops."""
    n_local, n_halo = cfg.n_local, cfg.n_halo
    n_cols = n_local + n_halo
    n_marg = min(n_local, cfg.n_send)
    n_central = n_local - n_marg

    deg = _degrees(rng, n_local, cfg.mean_degree, cap=max(1, n_local // 2), law=cfg.degree_law)
    draws = np.maximum(1, np.rint(deg * cfg.draw_inflation)).astype(np.int64)
    row_of_draw = np.repeat(np.arange(n_local, dtype=np.int64), draws)
    n_draw = int(row_of_draw.shape[0])

    halo_share = np.zeros(n_local, dtype=np.float64)
    halo_share[n_central:] = rng.uniform(0.30, 0.60, size=n_marg)
    to_halo = rng.random(n_draw) < halo_share[row_of_draw]

    draw_local = _popularity_sampler(rng, n_local)
    draw_halo = _popularity_sampler(rng, n_halo)
    u = rng.random(n_draw)
    cols = np.where(to_halo, n_local + draw_halo(u), draw_local(u))

    # self-loops for every row, and one guaranteed halo neighbour for every marginal row
    self_rows = np.arange(n_local, dtype=np.int64)
    marg_rows = np.arange(n_central, n_local, dtype=np.int64)
    forced_halo = n_local + draw_halo(rng.random(n_marg))
    rows_all = np.concatenate([row_of_draw, self_rows, marg_rows])
    cols_all = np.concatenate([cols, self_rows, forced_halo])

    key = np.unique(rows_all * n_cols + cols_all)       # removes duplicates, sorts by (row, col)
    rows_u = key // n_cols
    cols_u = (key - rows_u * n_cols).astype(np.int32)
    counts = np.bincount(rows_u, minlength=n_local).astype(np.int64)
    rowptr = np.zeros(n_local + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])

    # GCN symmetric normalisation: alpha(u, v) = 1 / sqrt(d~_u d~_v); d~ counts the self-loop.  For a halo
    # column (its true degree lives on another device) d~ is taken as 1 + the number of local rows citing it.
    d_row = counts.astype(np.float64)
    d_col = np.empty(n_cols, dtype=np.float64)
    d_col[:n_local] = d_row
    d_col[n_local:] = 1.0 + np.bincount(cols_u[cols_u >= n_local] - n_local, minlength=n_halo)
    if cfg.aggregator == "gcn":
        val = (1.0 / np.sqrt(d_row[rows_u] * d_col[cols_u])).astype(np.float32)
    elif cfg.aggregator == "mean":
        # mean aggregator (Sec. 5 trains GraphSAGE with it): every neighbour of a row, itself included, weighs 1/d~
        val = (1.0 / d_row[rows_u]).astype(np.float32)
    else:
        raise ValueError(cfg.aggregator)
    return rowptr, cols_u, val, n_central, n_cols


def _features(rng: np.random.Generator, kind: str, n: int, dim: int) -> np.ndarray:
    x = rng.standard_normal((n, dim), dtype=np.float32)
    if kind == "normal":
        return x
    if kind == "relu":
        return np.maximum(x, np.float32(0.0))
    if kind == "heavy_tail":
        cols = rng.choice(dim, size=min(50, dim), replace=False)
        x[:, cols] = rng.standard_t(3.0, size=(n, cols.shape[0])).astype(np.float32)
        return x
    if kind == "grad":
        return x * np.float32(1e-3)
    raise ValueError(kind)


def _peer_split(n_send: int, n_peers: int) -> np.ndarray:
    """Unbalanced slot counts per peer, proportional to 1/(p+1); every peer gets at least one slot."""
    w = 1.0 / np.arange(1, n_peers + 1, dtype=np.float64)
    cnt = np.floor(n_send * w / w.sum()).astype(np.int64)
    cnt = np.maximum(cnt, 1 if n_send >= n_peers else 0)
    cnt[0] += n_send - cnt.sum()
    return cnt


def _bits(rng: np.random.Generator, kind: str, n: int, score: Optional[np.ndarray]) -> np.ndarray:
    if kind == "uniform":
        return rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=n)
    if kind == "all2":
        return np.full(n, 2, dtype=np.uint8)
    if kind == "mix_c1":
        return rng.choice(np.array([4, 2, 8], dtype=np.uint8), size=n, p=[0.6, 0.3, 0.1])
    if kind == "adaptive":
        # stand-in for the assigner's output: the slots with the largest variance proxy get the widest codes
        order = np.argsort(-score, kind="stable")
        out = np.full(n, 2, dtype=np.uint8)
        out[order[: int(0.15 * n)]] = 8
        out[order[int(0.15 * n): int(0.60 * n)]] = 4
        return out
    raise ValueError(kind)


def make_partition(cfg: PartitionConfig, seed: Optional[int] = None) -> Partition:
    if seed is not None:
        cfg = replace(cfg, seed=seed)
    rng = np.random.default_rng(np.random.PCG64(cfg.seed))
    rowptr, col, val, n_central, n_cols = _forward_graph(rng, cfg)
    n_local, n_halo = cfg.n_local, cfg.n_halo
    cnt = _peer_split(cfg.n_send, cfg.n_peers)
    peer_of_slot = np.repeat(np.arange(cfg.n_peers, dtype=np.int32), cnt)

    if not cfg.backward:
        feat = _features(rng, cfg.feat, n_cols, cfg.dim)
        send_rows = n_central + rng.permutation(n_local - n_central)[: cfg.n_send]
        bits = _bits(rng, cfg.bits, cfg.n_send, None)
        halo_idx = (n_local + np.arange(cfg.n_send)).astype(np.int32)
        if cfg.n_send > n_halo:
            raise ValueError("loopback needs n_send <= n_halo")
        return Partition(cfg, rowptr, col, val, n_local, n_cols,
                         overlap_rows=(0, n_central), dependent_rows=(n_central, n_local),
                         n_central=n_central, feat=feat,
                         send_idx=send_rows.astype(np.int32), peer_of_slot=peer_of_slot, bits=bits,
                         halo_idx=halo_idx, meta={"direction": "forward"})

    # backward: hand out A^T (rows = local + halo nodes, columns = local nodes); the rows that are quantised
    # and sent back to their owners are the halo rows of A^T . dY
    import scipy.sparse as sp
    a = sp.csr_matrix((val, col, rowptr), shape=(n_local, n_cols))
    at = a.transpose().tocsr()
    at.sort_indices()
    t_rowptr = at.indptr.astype(np.int64)
    t_col = at.indices.astype(np.int32)
    t_val = at.data.astype(np.float32)
    dy = _features(rng, cfg.feat, n_local, cfg.dim)
    if cfg.n_send > n_halo:
        raise ValueError("backward needs n_send <= n_halo")
    send_rows = n_local + rng.permutation(n_halo)[: cfg.n_send]
    # variance proxy per slot: sum of squared coefficients of the edges feeding that gradient row
    sq = np.add.reduceat(np.square(t_val.astype(np.float64)), t_rowptr[:-1].clip(max=t_val.shape[0] - 1))
    sq[np.diff(t_rowptr) == 0] = 0.0
    bits = _bits(rng, cfg.bits, cfg.n_send, sq[send_rows])
    # loop-back stand-in for what the peers send back: every received slot carries the gradient of one of this
    # partition's marginal nodes; a peer names a node at most once, different peers may name the same node
    n_marg = n_local - n_central
    dst = np.concatenate([n_central + rng.permutation(n_marg)[:c] if c <= n_marg
                          else n_central + rng.integers(0, n_marg, size=c) for c in cnt]).astype(np.int32)
    return Partition(cfg, t_rowptr, t_col, t_val, n_cols, n_local,
                     overlap_rows=(0, n_local), dependent_rows=(n_local, n_cols),
                     n_central=n_central, feat=dy,
                     send_idx=send_rows.astype(np.int32), peer_of_slot=peer_of_slot, bits=bits,
                     halo_idx=dst, meta={"direction": "backward"})


def alpha_sq_stand_in(p: Partition) -> np.ndarray:
    """Input stand-in for the trace of Sec. 4.2: per send slot, the sum of squared aggregation coefficients the
    message meets on its target device.  That sum lives on the peer, which this one-partition workload does not
    have; the sum over the sending node's own CSR row takes its place (float32 [n_send], input slot order)."""
    sq = np.add.reduceat(np.square(p.val.astype(np.float64)), np.minimum(p.rowptr[:-1], max(p.nnz - 1, 0)))
    sq[np.diff(p.rowptr) == 0] = 0.0
    return sq[p.send_idx].astype(np.float32)
