"""Pins for the oracle's neighbour aggregation (Sec. 2.1 Eq. 3, inner sum) and the central/marginal split
(Sec. 3.1)."""
import numpy as np

from paper_2306_01381_amd.synth import CONFIGS, make_partition


def _random_csr(rng, n_rows, n_cols, density):
    dense = (rng.random((n_rows, n_cols)) < density) * rng.standard_normal((n_rows, n_cols))
    dense = dense.astype(np.float32)
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    col, val = [], []
    for r in range(n_rows):
        nz = np.nonzero(dense[r])[0]
        col += nz.tolist()
        val += dense[r, nz].tolist()
        rowptr[r + 1] = len(col)
    return dense, rowptr, np.array(col, np.int32), np.array(val, np.float32)


def test_matches_dense_brute_force(oracle):
    rng = np.random.default_rng(0)
    for n_rows, n_cols, dim, dens in [(1, 1, 1, 1.0), (17, 23, 5, 0.3), (64, 64, 33, 0.1), (40, 64, 130, 0.5)]:
        dense, rowptr, col, val = _random_csr(rng, n_rows, n_cols, dens)
        H = rng.standard_normal((n_cols, dim + 3), dtype=np.float32)            # ld > dim
        out = np.full((n_rows, dim + 1), np.float32(-5.0))
        out64, abs64 = oracle.spmm_csr(rowptr, col, val, 0, n_rows, H, dim, out=out)
        ref = dense.astype(np.float64) @ H[:, :dim].astype(np.float64)
        assert np.allclose(out64, ref, rtol=1e-12, atol=1e-12)
        assert np.array_equal(out[:, :dim], out64.astype(np.float32))
        assert np.all(out[:, dim] == -5.0)                                      # never writes past dim
        ref_abs = np.abs(dense.astype(np.float64)) @ np.abs(H[:, :dim].astype(np.float64))
        assert np.allclose(abs64, ref_abs, rtol=1e-12, atol=1e-12)


def test_row_range_only_touches_its_rows(oracle):
    rng = np.random.default_rng(1)
    dense, rowptr, col, val = _random_csr(rng, 30, 30, 0.2)
    H = rng.standard_normal((30, 8), dtype=np.float32)
    out = np.full((30, 8), np.float32(9.0))
    out64, _ = oracle.spmm_csr(rowptr, col, val, 11, 19, H, 8, out=out)
    ref = dense.astype(np.float64) @ H.astype(np.float64)
    assert np.all(out[:11] == 9.0) and np.all(out[19:] == 9.0)
    assert np.allclose(out64, ref[11:19], rtol=1e-12, atol=1e-12)
    out64e, _ = oracle.spmm_csr(rowptr, col, val, 7, 7, H, 8, out=out)
    assert out64e.shape == (0, 8)


def test_identity_stochastic_and_regular_graphs(oracle):
    rng = np.random.default_rng(2)
    n, dim = 50, 12
    H = rng.standard_normal((n, dim), dtype=np.float32)
    # A = I
    rowptr = np.arange(n + 1, dtype=np.int64)
    out = np.zeros((n, dim), np.float32)
    oracle.spmm_csr(rowptr, np.arange(n, dtype=np.int32), np.ones(n, np.float32), 0, n, H, dim, out=out)
    assert np.array_equal(out, H)
    # ring with self-loops, GCN weights: every node has 3 entries of 1/3 -> neighbourhood mean
    col = np.stack([(np.arange(n) - 1) % n, np.arange(n), (np.arange(n) + 1) % n], 1).astype(np.int32)
    val = np.full(3 * n, 1.0 / np.sqrt(3.0 * 3.0), dtype=np.float32)
    out64, _ = oracle.spmm_csr(np.arange(0, 3 * n + 1, 3, dtype=np.int64), col.reshape(-1), val, 0, n, H, dim)
    mean = (H[(np.arange(n) - 1) % n].astype(np.float64) + H + H[(np.arange(n) + 1) % n]) / 3
    assert np.allclose(out64, mean, rtol=1e-6)
    # row-stochastic matrix times the all-ones matrix gives ones
    dense = rng.random((n, n)) * (rng.random((n, n)) < 0.3)
    dense[np.arange(n), np.arange(n)] = 1.0
    dense /= dense.sum(1, keepdims=True)
    rp = np.zeros(n + 1, np.int64)
    c, v = [], []
    for r in range(n):
        nz = np.nonzero(dense[r])[0]
        c += nz.tolist()
        v += dense[r, nz].tolist()
        rp[r + 1] = len(c)
    out64, _ = oracle.spmm_csr(rp, np.array(c, np.int32), np.array(v, np.float32), 0, n,
                               np.ones((n, 4), np.float32), 4)
    assert np.allclose(out64, 1.0, rtol=1e-6)


def test_empty_rows_give_zero(oracle):
    rowptr = np.array([0, 0, 2, 2, 2], dtype=np.int64)
    out = np.full((4, 3), np.float32(4.0))
    H = np.arange(12, dtype=np.float32).reshape(4, 3)
    oracle.spmm_csr(rowptr, np.array([0, 3], np.int32), np.array([1.0, 2.0], np.float32), 0, 4, H, 3, out=out)
    assert np.array_equal(out[0], [0, 0, 0]) and np.array_equal(out[2], [0, 0, 0])
    assert np.array_equal(out[1], H[0] + 2 * H[3])


def test_central_rows_ignore_halo_contents(oracle):
    """Central nodes have no remote neighbour (Sec. 3.1), so their aggregate cannot depend on halo rows."""
    p = make_partition(CONFIGS["c0"])
    n_local = p.cfg.n_local
    assert p.n_central > 0
    assert p.col[: p.rowptr[p.n_central]].max() < n_local
    marg_has_halo = [p.col[p.rowptr[r]: p.rowptr[r + 1]].max() >= n_local for r in range(p.n_central, n_local)]
    assert all(marg_has_halo)
    a, _ = oracle.spmm_csr(p.rowptr, p.col, p.val, 0, p.n_central, p.feat, p.cfg.dim)
    poisoned = p.feat.copy()
    poisoned[n_local:] = np.nan
    b, _ = oracle.spmm_csr(p.rowptr, p.col, p.val, 0, p.n_central, poisoned, p.cfg.dim)
    assert np.array_equal(a, b)
    c, _ = oracle.spmm_csr(p.rowptr, p.col, p.val, p.n_central, n_local, poisoned, p.cfg.dim)
    assert np.isnan(c).any(axis=1).all()
