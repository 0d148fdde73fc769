"""adaqp_spmm_csr_noalloc (the aggregation with the library's built-in scratch, for callers that cannot allocate)
against adaqp_spmm_csr with a caller-provided workspace, through the C ABI: two calls in a row on the same GPU, the
second on a smaller input, so that the second finds the first one's leftovers in the shared scratch."""
import ctypes
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2306_01381_amd import binding as B                      # noqa: E402

DEV = "cuda:0"
SPMM_RTOL = 1e-5


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.lib()


def _graph(rng, n_rows, n_cols, mean_deg):
    deg = np.minimum(rng.zipf(1.6, size=n_rows) * mean_deg // 3 + 1, n_cols).astype(np.int64)
    deg[rng.integers(0, n_rows, size=max(1, n_rows // 50))] = 0            # some empty rows
    deg[rng.integers(0, n_rows)] = min(n_cols, 40 * mean_deg)              # one row split over many pieces
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    col = np.concatenate([np.sort(rng.choice(n_cols, size=int(d), replace=False)) for d in deg]).astype(np.int32)
    val = rng.standard_normal(col.shape[0]).astype(np.float32)
    return rowptr, col, val


def _both(rowptr, col, val, rb, re, H, dim, ldo):
    """(out of adaqp_spmm_csr, out of adaqp_spmm_csr_noalloc) for rows [rb, re), sentinel elsewhere."""
    t_rowptr, t_col, t_val = (torch.from_numpy(a).to(DEV) for a in (rowptr, col, val))
    t_H = torch.from_numpy(H).to(DEV)
    n_rows = rowptr.shape[0] - 1
    nnz_range = int(rowptr[re] - rowptr[rb])
    ws = torch.empty(max(B.adaqp_spmm_workspace_bytes(re - rb, nnz_range, dim), 256), dtype=torch.uint8, device=DEV)
    want = torch.full((n_rows, ldo), 7.0, dtype=torch.float32, device=DEV)
    got = torch.full((n_rows, ldo), 7.0, dtype=torch.float32, device=DEV)
    B.adaqp_spmm_csr(t_rowptr, t_col, t_val, rb, re, t_H[:, :dim] if H.shape[1] != dim else t_H, dim,
                     want[:, :dim] if ldo != dim else want, ws, nnz_range=nnz_range)
    torch.cuda.synchronize()
    # nothing below may allocate device memory inside the library: the call takes no workspace
    B.adaqp_spmm_csr_noalloc(t_rowptr, t_col, t_val, rb, re, t_H[:, :dim] if H.shape[1] != dim else t_H, dim,
                             got[:, :dim] if ldo != dim else got, nnz_range=nnz_range)
    torch.cuda.synchronize()
    return want.cpu().numpy(), got.cpu().numpy()


def test_noalloc_aggregation_matches_the_workspace_entry_point(oracle):
    rng = np.random.default_rng(2306)
    # first call: 3000 rows of 602 columns (line-padded pitch 608); second: a smaller graph, other width, a row range
    cases = [(3000, 4100, 24, 602, 608, 0, 3000), (700, 900, 9, 130, 160, 100, 650)]
    for n_rows, n_cols, mean_deg, dim, ld, rb, re in cases:
        _say(f"noalloc spmm: rows={n_rows} cols={n_cols} dim={dim} ld={ld} range=[{rb},{re})")
        rowptr, col, val = _graph(rng, n_rows, n_cols, mean_deg)
        H = rng.standard_normal((n_cols, ld), dtype=np.float32)
        want, got = _both(rowptr, col, val, rb, re, H, dim, ld)
        # same kernels, same launch geometry: the same bits, in the rows of the range and (sentinel) outside it
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
        # and both within the aggregation's bar of the fp64 oracle
        Hc = np.ascontiguousarray(H)
        ref, mag = oracle.spmm_csr(rowptr, col, val, rb, re, Hc, dim)
        err = np.abs(got[rb:re, :dim].astype(np.float64) - ref)
        assert np.all(err <= SPMM_RTOL * mag + 1e-30)
        assert np.all(got[:rb] == 7.0) and np.all(got[re:] == 7.0)


def test_noalloc_rejects_what_does_not_fit_its_scratch():
    L = B.lib()
    need = B.adaqp_spmm_workspace_bytes(60000, 30_000_000, 602)
    assert need > B.SPMM_NOALLOC_SCRATCH_BYTES
    one = torch.zeros(256, dtype=torch.uint8, device=DEV)           # valid, aligned pointers; nothing is launched
    p = one.data_ptr()
    rc = L.adaqp_spmm_csr_noalloc(p, p, p, 30_000_000, 0, 60000, -1, p, 98000, 608, 602, p, 608, None)
    assert rc == B.ESIZE
    assert L.adaqp_spmm_csr_noalloc(None, p, p, 10, 0, 5, -1, p, 10, 8, 8, p, 8, None) == B.EINVAL
    assert L.adaqp_spmm_csr_noalloc(p, p, p, 10, 0, 0, -1, p, 10, 8, 8, p, 8, None) == B.OK       # no rows: no-op
