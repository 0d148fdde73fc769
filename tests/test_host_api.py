"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host logic
(layout planning, argument validation that happens before any launch) behaves as the header says."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2306_01381_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for header in sorted(os.listdir(inc)):
        if header.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, header)).read(), flags=re.S)
            names |= set(re.findall(r"\b(adaqp_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared_symbols()
    assert len(names) >= 10
    for n in names:
        assert hasattr(L, n), n
    assert set(names) == set(B.EXPORTS)
    assert B.adaqp_version() >= 100
    assert L.adaqp_strerror(B.ESIZE).decode().startswith("buffer")


def test_row_stride():
    assert B.adaqp_row_stride(602, 2) == 152 and B.adaqp_row_stride(602, 4) == 304
    assert B.adaqp_row_stride(602, 8) == 604 and B.adaqp_row_stride(1, 2) == 4
    assert B.adaqp_row_stride(256, 2) == 64
    assert B.adaqp_row_stride(0, 2) == -1 and B.adaqp_row_stride(8, 3) == -1


def test_plan_layout_matches_oracle(oracle):
    rng = np.random.default_rng(4)
    for dim in (1, 5, 128, 300, 602, 4100):
        for n, n_peers in ((0, 2), (1, 1), (37, 3), (500, 7)):
            peer = np.sort(rng.integers(0, n_peers, size=n)).astype(np.int32)
            bits = rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=n)
            got = B.adaqp_plan_layout(dim, bits, peer, n_peers)
            want = oracle.plan_layout(dim, bits, peer, n_peers)
            for g, w in zip(got, want):
                assert np.array_equal(g, w)


def test_plan_layout_errors():
    with pytest.raises(B.AdaqpError) as e:
        B.adaqp_plan_layout(8, np.array([2, 5], np.uint8), np.array([0, 0], np.int32), 1)
    assert e.value.status == B.EBITS
    with pytest.raises(B.AdaqpError) as e:
        B.adaqp_plan_layout(8, np.array([2, 2], np.uint8), np.array([1, 0], np.int32), 2)
    assert e.value.status == B.EINVAL
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_layout(0, np.array([2], np.uint8), np.array([0], np.int32), 1)
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_layout(8, np.array([2], np.uint8), np.array([3], np.int32), 3)


def test_argument_errors_are_caught_before_any_launch():
    L = B.lib()
    one = ctypes.c_void_p(256)          # a non-NULL, aligned dummy; never dereferenced on these paths
    # zero counts are successful no-ops
    assert L.adaqp_quantize_pack(None, 0, 8, 8, None, None, None, 0, 0, None, 0, None, None) == B.OK
    assert L.adaqp_unpack_dequant(None, 0, None, None, None, None, None, 0, 8, None, 0, 8, None) == B.OK
    assert L.adaqp_spmm_csr(None, None, None, 0, 3, 3, -1, None, 0, 8, 8, None, 8, None, 0, None) == B.OK
    # bad shapes
    assert L.adaqp_quantize_pack(one, 4, 7, 8, one, one, one, 1, 0, one, 64, one, None) == B.EINVAL   # ld < dim
    assert L.adaqp_quantize_pack(one, 4, 8, 0, one, one, one, 1, 0, one, 64, one, None) == B.EINVAL   # dim 0
    assert L.adaqp_quantize_pack(one, 4, 8, 8, one, one, one, -1, 0, one, 64, one, None) == B.EINVAL  # n < 0
    assert L.adaqp_quantize_pack(None, 4, 8, 8, one, one, one, 1, 0, one, 64, one, None) == B.EINVAL  # NULL
    assert L.adaqp_unpack_dequant(one, 64, one, one, one, one, None, 1, 8, None, 4, 8, None) == B.EINVAL
    assert L.adaqp_unpack_dequant(one, 64, one, one, one, one, None, 1, 8, one, 4, 4, None) == B.EINVAL  # ld < dim
    assert L.adaqp_spmm_csr(one, one, one, 5, 2, 1, -1, one, 4, 8, 8, one, 8, one, 1 << 20, None) == B.EINVAL
    assert L.adaqp_spmm_csr(one, one, one, 5, 0, 2, -1, one, 4, 4, 8, one, 8, one, 1 << 20, None) == B.EINVAL
    # workspace too small
    assert L.adaqp_spmm_csr(one, one, one, 5, 0, 2, -1, one, 4, 8, 8, one, 8, one, 16, None) == B.ESIZE
    assert L.adaqp_layer_step(None) == B.EINVAL
    d = B.LayerDesc()
    d.direction = 7
    assert L.adaqp_layer_step(ctypes.byref(d)) == B.EINVAL
    # panels: nothing to do is fine, anything inconsistent is refused on the host
    assert L.adaqp_spmm_csr_panels(None, 0, 4, one, 8, 32, 8, one, 32, one, 1 << 20, None) == B.EINVAL
    none = B.SpmmPanels()
    assert L.adaqp_spmm_csr_panels(ctypes.byref(none), 0, 4, one, 8, 32, 8, one, 32, one, 1 << 20, None) == B.OK
    some = B.SpmmPanels(1, 1, 1, 1, 256, 256, 256, 256, 256, 256)
    assert L.adaqp_spmm_csr_panels(ctypes.byref(some), 0, 4, one, 8, 32, 8, one, 32, one, 16, None) == B.ESIZE
    assert L.adaqp_spmm_csr_panels(ctypes.byref(some), 0, 4, one, 8, 24, 8, one, 32, one, 1 << 20, None) == B.EINVAL  # pitch
    assert L.adaqp_spmm_csr_panels(ctypes.byref(some), 0, 4, one, 8, 32, 8, one, 32, None, 1 << 20, None) == B.EINVAL
    assert L.adaqp_spmm_csr_panels(ctypes.byref(some), 4, 0, one, 8, 32, 8, one, 32, one, 1 << 20, None) == B.EINVAL
    holes = B.SpmmPanels(1, 1, 1, 1, 256, 0, 256, 256, 256, 256)                    # an array missing
    assert L.adaqp_spmm_csr_panels(ctypes.byref(holes), 0, 4, one, 8, 32, 8, one, 32, one, 1 << 20, None) == B.EINVAL
    many = B.SpmmPanels(1, 1, 1, 9, 256, 256, 256, 256, 256, 256)                   # more pieces than piece slots
    assert L.adaqp_spmm_csr_panels(ctypes.byref(many), 0, 4, one, 8, 32, 8, one, 32, one, 1 << 20, None) == B.EINVAL
    bad = B.SpmmPanels(-1, 0, 0, 0, 0, 0, 0, 0, 0, 0)
    assert L.adaqp_spmm_csr_panels(ctypes.byref(bad), 0, 4, one, 8, 32, 8, one, 32, one, 1 << 20, None) == B.EINVAL


def test_workspace_query():
    assert B.adaqp_spmm_workspace_bytes(0, 0, 8) == 0
    small = B.adaqp_spmm_workspace_bytes(2000, 20000, 128)
    big = B.adaqp_spmm_workspace_bytes(58000, 28_000_000, 602)
    assert small % 256 == 0 and big % 256 == 0 and 0 < small < big < (1 << 30)
    with pytest.raises(B.AdaqpError):
        B.adaqp_spmm_workspace_bytes(-1, 0, 8)


def test_plan_recv_order():
    rng = np.random.default_rng(3)
    halo = rng.permutation(5000)[:700].astype(np.int32) + 100
    order = B.adaqp_plan_recv_order(halo)
    assert order.dtype == np.int32 and sorted(order.tolist()) == list(range(700))
    assert np.all(np.diff(halo[order]) > 0)
    assert np.array_equal(order, np.argsort(halo, kind="stable"))
    assert B.adaqp_plan_recv_order(np.zeros(0, np.int32)).size == 0
    # ties keep slot order
    assert B.adaqp_plan_recv_order(np.array([5, 1, 5, 1], np.int32)).tolist() == [1, 3, 0, 2]


def test_plan_recv_segments():
    dst = np.array([7, 3, 7, 9, 3, 3], dtype=np.int32)
    order, seg_ptr = B.adaqp_plan_recv_segments(dst)
    assert order.tolist() == [1, 4, 5, 0, 2, 3]              # by destination, slot order inside
    assert seg_ptr.tolist() == [0, 3, 5, 6]
    order, seg_ptr = B.adaqp_plan_recv_segments(np.zeros(0, np.int32))
    assert order.size == 0 and seg_ptr.tolist() == [0]
    rng = np.random.default_rng(8)
    dst = rng.integers(0, 300, size=2000).astype(np.int32)
    order, seg_ptr = B.adaqp_plan_recv_segments(dst)
    assert sorted(order.tolist()) == list(range(2000))
    assert np.all(np.diff(dst[order]) >= 0)
    assert len(seg_ptr) - 1 == len(np.unique(dst))
    for g in range(len(seg_ptr) - 1):
        seg = order[seg_ptr[g]: seg_ptr[g + 1]]
        assert len(set(dst[seg].tolist())) == 1 and np.all(np.diff(seg) > 0)


def test_plan_slot_of_row():
    halo = np.array([7, 3, 9, 4], dtype=np.int32)
    m = B.adaqp_plan_slot_of_row(10, halo)
    assert m.dtype == np.int32 and m.tolist() == [-1, -1, -1, 1, 3, -1, -1, 0, -1, 2]
    assert B.adaqp_plan_slot_of_row(3, np.zeros(0, np.int32)).tolist() == [-1, -1, -1]
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_slot_of_row(10, np.array([1, 1], dtype=np.int32))       # a row listed twice
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_slot_of_row(10, np.array([10], dtype=np.int32))         # out of range


def test_plan_spmm_tiles():
    rng = np.random.default_rng(3)
    n_rows, n_cols = 40, 100
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    cols = []
    for r in range(n_rows):
        d = int(rng.integers(0, 30)) if r % 3 else int(rng.integers(64, 100))      # short and long rows
        cols.append(np.sort(rng.choice(n_cols, size=d, replace=False)))
        rowptr[r + 1] = rowptr[r] + d
    col = np.concatenate(cols).astype(np.int32)
    bounds, off = B.adaqp_plan_spmm_tiles(rowptr, col, 0, n_rows, n_cols)
    assert bounds.shape == (B.SPMM_TILES + 1,) and off.shape == (n_rows, B.SPMM_TILES + 1)
    assert bounds[0] == 0 and bounds[-1] == col.max() + 1 and np.all(np.diff(bounds) >= 0)
    def want_row(r, first_row, c, bnd):
        if len(c) >= B.SPMM_TILED_SHORT_ROW:
            return [int(np.count_nonzero(c < b)) for b in bnd]
        home = (r - first_row) % B.SPMM_TILES                      # a short row stays whole, in one tile
        return [0 if t <= home else len(c) for t in range(B.SPMM_TILES + 1)]

    for r in range(n_rows):
        assert off[r].tolist() == want_row(r, 0, col[rowptr[r]: rowptr[r + 1]], bounds)
    per_tile = np.array([np.count_nonzero((col >= bounds[t]) & (col < bounds[t + 1])) for t in range(B.SPMM_TILES)])
    uses = np.bincount(col, minlength=n_cols)
    assert per_tile.sum() == len(col)
    assert np.all(np.abs(per_tile - len(col) / B.SPMM_TILES) <= uses.max() + 1)      # equal up to one column's uses
    # a sub-range is planned from its own entries and indexed from its first row
    b2, off2 = B.adaqp_plan_spmm_tiles(rowptr, col, 10, 25, n_cols)
    assert off2.shape == (15, B.SPMM_TILES + 1)
    for r in (12, 13, 14, 15):
        assert off2[r - 10].tolist() == want_row(r, 10, col[rowptr[r]: rowptr[r + 1]], b2)
    # empty range, empty graph
    b3, off3 = B.adaqp_plan_spmm_tiles(rowptr, col, 5, 5, n_cols)
    assert off3.shape == (0, B.SPMM_TILES + 1) and b3[-1] == 0
    assert B.adaqp_spmm_tiled_workspace_bytes(10, 602) == 8 * 10 * 608 * 4
    assert B.adaqp_spmm_tiled_pays(28000, 12_763_658) and B.adaqp_spmm_tiled_pays(30000, 15_478_947)   # c1
    assert not B.adaqp_spmm_tiled_pays(306000, 7_680_000) and not B.adaqp_spmm_tiled_pays(0, 0)          # c2, empty
    # chunk width: 128 columns while the widest column range x 512 B stays within about 5 MB
    even = np.arange(9, dtype=np.int32)
    assert B.adaqp_spmm_tiled_chunk_cols(even * 7000, 602) == 128
    assert B.adaqp_spmm_tiled_chunk_cols(even * 13000, 602) == 64
    assert B.adaqp_spmm_tiled_chunk_cols(even * 7000, 64) == 64
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_spmm_tiles(np.array([0, 2], np.int64), np.array([5, 5], np.int32), 0, 1, 8)   # repeated column


def _panel_csr(seed, n_rows=90, n_cols=300):
    rng = np.random.default_rng(seed)
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    cols = []
    for r in range(n_rows):
        d = int(rng.integers(0, 20)) if r % 2 else int(rng.integers(40, 200))           # short and long rows
        cols.append(np.sort(rng.choice(n_cols, size=d, replace=False)))
        rowptr[r + 1] = rowptr[r] + d
    col = np.concatenate(cols).astype(np.int32)
    val = rng.standard_normal(len(col)).astype(np.float32)
    val[val == 0] = 1.0
    return rowptr, col, val


def _decode_panels(plan, n_cols):
    """Dense [n_panels * 32, n_cols] matrix a panel plan stands for, every piece visited once through the
    per-panel piece lists; also the tile of every piece."""
    dense = np.zeros((plan["n_panels"] * B.SPMM_PANEL_ROWS, n_cols), dtype=np.float64)
    npt = plan["n_per_tile"]
    seen = set()
    for p in range(plan["n_panels"]):
        ids = plan["panel_piece"][plan["panel_piece_ptr"][p]: plan["panel_piece_ptr"][p + 1]]
        assert np.all(np.diff(ids) > 0)                                 # ascending: the summation order
        for pid in ids:
            assert pid not in seen
            seen.add(int(pid))
            g0, g1 = plan["piece"][pid // npt, pid % npt]
            assert 0 <= g0 < g1 <= plan["n_groups"]
            for g in range(g0, g1):
                for u in range(4):
                    for h in range(2):
                        c = plan["pcol"][g, h, u]
                        dense[p * 32: p * 32 + 32, c] += plan["palpha"][g, 32 * h: 32 * h + 32, u]
    return dense, seen


def test_plan_spmm_panels():
    n_cols = 300
    rowptr, col, val = _panel_csr(11, n_cols=n_cols)
    n_rows = len(rowptr) - 1
    for (rb, re, min_len, piece_cols) in ((0, n_rows, 40, 16), (7, 61, 100, 8), (0, n_rows, 150, 1024)):
        bounds, off = B.adaqp_plan_spmm_tiles(rowptr, col, rb, re, n_cols)
        off0 = off.copy()
        plan = B.adaqp_plan_spmm_panels(rowptr, col, val, rb, re, n_cols, bounds, off, min_len, piece_cols)
        deg = np.diff(rowptr)
        want_rows = [r for r in range(rb, re) if deg[r] >= min_len]
        want_rows.sort(key=lambda r: (-deg[r], r))
        assert plan["n_rows_taken"] == len(want_rows) and plan["n_panels"] == (len(want_rows) + 31) // 32
        rows = plan["panel_rows"]
        assert rows[: len(want_rows)].tolist() == want_rows and np.all(rows[len(want_rows):] == -1)
        dense, seen = _decode_panels(plan, n_cols)
        assert len(seen) == plan["n_panel_pieces"]
        for k, r in enumerate(rows):
            want = np.zeros(n_cols)
            if r >= 0:
                want[col[rowptr[r]: rowptr[r + 1]]] = val[rowptr[r]: rowptr[r + 1]]
            assert np.array_equal(dense[k], want), (k, r)
        # pieces of tile t stay inside the tile's column range (the last tile takes the rest), within piece_cols
        npt = plan["n_per_tile"]
        used = 0
        for t in range(B.SPMM_TILES):
            for i in range(npt):
                g0, g1 = plan["piece"][t, i]
                if g0 == g1:
                    continue
                used += 1
                assert (g1 - g0) * 8 <= piece_cols
                c = plan["pcol"][g0:g1].reshape(-1)
                assert c.min() >= bounds[t] and (t == B.SPMM_TILES - 1 or c.max() < bounds[t + 1])
        assert used == plan["n_panel_pieces"]
        # the pieces of one (panel, tile): as few as piece_cols allows, equal in size to within one group
        sizes = {}
        for p_ in range(plan["n_panels"]):
            for pid in plan["panel_piece"][plan["panel_piece_ptr"][p_]: plan["panel_piece_ptr"][p_ + 1]]:
                g0, g1 = plan["piece"][pid // npt, pid % npt]
                sizes.setdefault((p_, int(pid) // npt), []).append(int(g1 - g0))
        for key, sz in sizes.items():
            assert max(sz) - min(sz) <= 1, (key, sz)
            assert len(sz) == -(-sum(sz) // (piece_cols // 8)), (key, sz)
        # the rows taken are struck from the tile table, the others are untouched
        taken = np.zeros(re - rb, dtype=bool)
        taken[np.array(want_rows, dtype=np.int64) - rb] = True
        assert np.all(off[taken] == -1) and np.array_equal(off[~taken], off0[~taken])
    # nothing long enough: no plan, table untouched
    bounds, off = B.adaqp_plan_spmm_tiles(rowptr, col, 0, n_rows, n_cols)
    off0 = off.copy()
    assert B.adaqp_plan_spmm_panels(rowptr, col, val, 0, n_rows, n_cols, bounds, off, 1000) is None
    assert np.array_equal(off, off0)
    assert B.adaqp_spmm_panels_workspace_bytes(218, 602) == 8 * 218 * 32 * 608 * 4
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_spmm_panels(rowptr, col, val, 0, n_rows, n_cols, bounds, None, 40, 12)     # piece_cols % 8
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_spmm_panels(rowptr, col, val, 0, n_rows, n_cols, bounds, None, 0, 16)      # min_row_len < 1
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_spmm_panels(np.array([0, 2], np.int64), np.array([5, 5], np.int32), np.ones(2, np.float32),
                                 0, 1, 8, np.zeros(9, np.int32), None, 1, 8)                    # repeated column


def test_plan_spmm_panels_random_graphs():
    """Seeded sweep: whatever the shape, the plan decodes back to exactly the rows it took."""
    rng = np.random.default_rng(2024)
    for case in range(12):
        n_rows = int(rng.choice([1, 5, 33, 64, 130]))
        n_cols = int(rng.choice([1, 7, 8, 9, 40, 257]))
        degs = rng.integers(0, n_cols + 1, size=n_rows)
        if case % 3 == 0:
            degs[:] = n_cols                                            # dense
        rowptr = np.zeros(n_rows + 1, dtype=np.int64)
        cols = []
        for r in range(n_rows):
            cols.append(np.sort(rng.choice(n_cols, size=int(degs[r]), replace=False)))
            rowptr[r + 1] = rowptr[r] + degs[r]
        col = np.concatenate(cols).astype(np.int32)
        val = (rng.standard_normal(len(col)) + 3.0).astype(np.float32)  # never zero
        rb = int(rng.integers(0, n_rows))
        re = int(rng.integers(rb, n_rows + 1))
        min_len = int(rng.choice([1, 2, 5, 30]))
        piece_cols = int(rng.choice([8, 16, 64]))
        bounds, off = B.adaqp_plan_spmm_tiles(rowptr, col, rb, re, n_cols)
        plan = B.adaqp_plan_spmm_panels(rowptr, col, val, rb, re, n_cols, bounds, off, min_len, piece_cols)
        want_rows = [r for r in range(rb, re) if degs[r] >= min_len]
        if not want_rows:
            assert plan is None, case
            continue
        assert sorted(plan["panel_rows"][plan["panel_rows"] >= 0].tolist()) == want_rows, case
        dense, seen = _decode_panels(plan, n_cols)
        assert len(seen) == plan["n_panel_pieces"], case
        for k, r in enumerate(plan["panel_rows"]):
            want = np.zeros(n_cols)
            if r >= 0:
                want[col[rowptr[r]: rowptr[r + 1]]] = val[rowptr[r]: rowptr[r + 1]]
            assert np.array_equal(dense[k], want), (case, k, r)


def test_rule_that_decides_whether_a_panel_plan_pays():
    # one wave per (piece, 128-column chunk); fewer than ADAQP_SPMM_PANEL_MIN_WAVES of them do not fill the GPU
    assert not B.adaqp_spmm_panels_pay(0, 602) and not B.adaqp_spmm_panels_pay(100, 0)
    assert not B.adaqp_spmm_panels_pay(60, 602)            # one panel of a 602-column graph: 300 waves
    assert B.adaqp_spmm_panels_pay(1150, 602)              # eighteen panels: 5750 waves
    assert B.adaqp_spmm_panels_pay(2048, 128) and not B.adaqp_spmm_panels_pay(2047, 128)
    assert B.adaqp_spmm_panels_pay(410, 602) and not B.adaqp_spmm_panels_pay(409, 602)      # 5 chunks per piece
    # the planner binding turns a sized plan down on request and then leaves the tile table alone
    rng = np.random.default_rng(4)
    n_rows, n_cols = 40, 300
    degs = np.full(n_rows, 5)
    degs[:3] = 200
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(degs, out=rowptr[1:])
    col = np.concatenate([np.sort(rng.choice(n_cols, size=d, replace=False)) for d in degs]).astype(np.int32)
    val = rng.standard_normal(col.shape[0]).astype(np.float32)
    bounds, off = B.adaqp_plan_spmm_tiles(rowptr, col, 0, n_rows, n_cols)
    before = off.copy()
    assert B.adaqp_plan_spmm_panels(rowptr, col, val, 0, n_rows, n_cols, bounds, off, 100, 64,
                                    only_if_pays_for_dim=128) is None
    assert np.array_equal(off, before)
    assert B.adaqp_plan_spmm_panels(rowptr, col, val, 0, n_rows, n_cols, bounds, off, 100, 64) is not None
    assert not np.array_equal(off, before)


def test_layer_desc_mirror_matches_the_library():
    import ctypes
    assert int(B.lib().adaqp_layer_desc_bytes()) == ctypes.sizeof(B.LayerDesc)
