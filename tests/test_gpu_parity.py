"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars: packed bytes, (Z, S) and de-quantised fp32 values bit-exact; aggregation within
1e-5 * sum|terms| per output element (the fp64 oracle also returns that sum).
"""
import sys
from dataclasses import replace

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2306_01381_amd import binding as B                      # noqa: E402
from paper_2306_01381_amd.layer import LayerStep, SendPlan          # noqa: E402
from paper_2306_01381_amd.synth import CONFIGS, make_partition      # noqa: E402

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


def _gpu_quantize(feat_np, dim, send_idx, bits, off, seed, packed_bytes, fill=0xAB):
    feat = torch.from_numpy(feat_np).to(DEV)
    packed = torch.full((max(packed_bytes, 4),), fill, dtype=torch.uint8, device=DEV)
    params = torch.full((max(len(send_idx), 1), 2), float("nan"), dtype=torch.float32, device=DEV)
    B.adaqp_quantize_pack(feat, dim, torch.from_numpy(send_idx).to(DEV), torch.from_numpy(bits).to(DEV),
                          torch.from_numpy(off).to(DEV), seed, packed, params)
    torch.cuda.synchronize()
    return packed.cpu().numpy(), params.cpu().numpy()


def _padded_cols(dim, ld):
    """Columns a line-padded output row gets zero-filled (torch allocations are at least 256-byte aligned)."""
    return min(ld, (dim + 31) // 32 * 32) if ld % 32 == 0 else dim


def _codec_case(oracle, feat_np, dim, send_idx, bits, peer, n_peers, seed, halo_rows=None, use_order=False):
    """Quantise on both sides, compare bytes and params; de-quantise on both sides, compare floats."""
    perm, off, pbp = oracle.plan_layout(dim, bits, peer, n_peers)
    perm_g, off_g, pbp_g = B.adaqp_plan_layout(dim, bits, peer, n_peers)
    assert np.array_equal(perm, perm_g) and np.array_equal(off, off_g) and np.array_equal(pbp, pbp_g)
    s_idx = np.ascontiguousarray(send_idx[perm], dtype=np.int32)
    s_bits = np.ascontiguousarray(bits[perm], dtype=np.uint8)
    nbytes = int(pbp[-1])
    want_packed, want_params, _ = oracle.quantize_pack(feat_np, dim, s_idx, s_bits, off, seed, nbytes)
    got_packed, got_params = _gpu_quantize(feat_np, dim, s_idx, s_bits, off, seed, nbytes)
    n = len(s_idx)
    assert np.array_equal(got_params[:n].view(np.uint32), want_params.view(np.uint32)), "(Z, S) differ"
    if nbytes:
        bad = np.nonzero(got_packed[:nbytes] != want_packed)[0]
        assert bad.size == 0, f"{bad.size} packed bytes differ, first at {bad[:5]}"
    # receive side, into a copy with a sentinel so that stray writes show
    ld = feat_np.shape[1]
    n_rows = feat_np.shape[0]
    halo = np.ascontiguousarray(halo_rows if halo_rows is not None
                                else np.random.default_rng(seed).permutation(n_rows)[:n], dtype=np.int32)
    want = np.full((n_rows, ld), np.float32(-123.5))
    oracle.unpack_dequant(want_packed, want_params, s_bits, off, halo, dim, want)
    want[halo, dim:_padded_cols(dim, ld)] = 0.0            # whole-line writes zero the row padding
    got = torch.full((n_rows, ld), -123.5, dtype=torch.float32, device=DEV)
    order = torch.from_numpy(B.adaqp_plan_recv_order(halo)).to(DEV) if use_order else None
    B.adaqp_unpack_dequant(torch.from_numpy(want_packed if nbytes else np.zeros(4, np.uint8)).to(DEV),
                           torch.from_numpy(want_params if n else np.zeros((1, 2), np.float32)).to(DEV),
                           torch.from_numpy(s_bits).to(DEV), torch.from_numpy(off).to(DEV),
                           torch.from_numpy(halo).to(DEV), dim, got, order=order)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32)), "de-quantised rows differ"


@pytest.mark.parametrize("dim,ld", [(128, 128), (602, 602), (256, 256), (300, 300), (300, 301), (7, 7), (1, 1),
                                    (8, 12), (9, 9), (33, 40), (63, 63), (64, 64), (65, 66), (1000, 1000),
                                    (4096, 4096), (4100, 4100), (5000, 5001),
                                    # line-padded pitches: whole-line reads and writes, ragged last vector
                                    (602, 608), (300, 320), (7, 32), (33, 64), (1, 32), (130, 160), (1000, 1024),
                                    (250, 256), (2047, 2048), (2049, 2080), (4100, 4128), (602, 640), (602, 604)])
def test_codec_shapes(oracle, dim, ld):
    _say(f"codec dim={dim} ld={ld}")
    rng = np.random.default_rng(dim * 7 + ld)
    n_rows, n = 300, 211                       # several blocks of rows and a ragged last block
    feat = rng.standard_normal((n_rows, ld), dtype=np.float32)
    feat[:, dim:] = np.float32(1e30)           # padding must never enter min / max
    feat[3] = 1.25                                                    # constant row
    feat[4, : dim // 2] = 0.0
    feat[5] = np.maximum(feat[5], 0)
    feat[6] *= np.float32(1e-3)
    send = rng.integers(0, n_rows, size=n).astype(np.int32)
    send[:8] = np.arange(8)
    bits = rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=n)
    peer = np.sort(rng.integers(0, 3, size=n)).astype(np.int32)
    _codec_case(oracle, feat, dim, send, bits, peer, 3, seed=dim, use_order=(dim % 2 == 0))


@pytest.mark.parametrize("b", [2, 4, 8])
def test_codec_single_width_and_seeds(oracle, b):
    _say(f"codec single width b={b}")
    rng = np.random.default_rng(b)
    feat = rng.standard_normal((64, 602), dtype=np.float32)
    for seed in (0, 1, 2**32 + 5, 2**64 - 1):
        _codec_case(oracle, feat, 602, np.arange(64, dtype=np.int32), np.full(64, b, np.uint8),
                    np.zeros(64, np.int32), 1, seed)


@pytest.mark.parametrize("dim,ld", [(24, 24), (602, 608), (300, 320), (5000, 5000)])
def test_codec_tiny_ranges_and_signed_zeros(oracle, dim, ld):
    """Rows at the bottom of fp32 (ranges from 1e-30 down to the smallest denormal: the scale with the 2^16 folded
    in overflows, then the reciprocal itself), rows whose minimum is reached by both -0.0 and +0.0, constant rows
    of either zero - next to ordinary rows in the same waves, every width."""
    _say(f"codec tiny ranges dim={dim} ld={ld}")
    rng = np.random.default_rng(dim)
    scales = [1.0, 1e-30, 1e-33, 1e-36, 3e-38, 1e-39, 1e-42, 3e-45, 1e-3]
    n_rows = 6 * len(scales)
    feat = np.zeros((n_rows, ld), dtype=np.float32)
    for i, sc in enumerate(scales):
        u = rng.random((6, dim))
        u[:, 0], u[:, -1] = 0.0, 1.0
        base = np.array([0.0, sc * 8, -sc * 3, 1e-20, 0.0, 0.0])[:, None]
        rows = (base + u * sc).astype(np.float32)
        rows[4] = np.float32(sc)
        rows[5, 1:] = rows[5, 0]
        if dim > 1:
            rows[5, 1] = np.nextafter(rows[5, 0], np.float32(1), dtype=np.float32)
        feat[6 * i: 6 * i + 6, :dim] = rows
    zeros = np.zeros((6, ld), dtype=np.float32)
    zeros[0, :dim] = np.maximum(rng.standard_normal(dim), 0)      # ReLU-like row: minimum +0.0 ...
    zeros[0, dim // 2] = -0.0                                      # ... and -0.0
    zeros[0, 0] = 0.0
    zeros[1, :dim] = -np.maximum(rng.standard_normal(dim), 0)     # maximum reached by both zeros
    zeros[1, 0] = 0.0
    zeros[1, dim - 1] = -0.0
    zeros[2, :dim] = -0.0                                          # constant -0.0
    zeros[3, :dim] = 0.0
    zeros[3, dim - 1] = -0.0                                       # "constant" row holding both zeros
    zeros[4, :dim] = rng.standard_normal(dim).astype(np.float32)
    zeros[5, :dim] = np.where(rng.random(dim) < 0.5, 0.0, -0.0)   # a mixture of the two zeros only
    feat = np.concatenate([feat, zeros], 0)
    n_rows = feat.shape[0]                                         # the rows that are sent
    feat = np.concatenate([feat, rng.standard_normal((2 * n_rows, ld), dtype=np.float32)], 0)   # room to receive
    feat[:, dim:] = np.float32(1e30)
    for b in (2, 4, 8):
        send = np.concatenate([np.arange(n_rows), rng.permutation(n_rows)]).astype(np.int32)
        bits = np.full(send.shape[0], b, np.uint8)
        _codec_case(oracle, feat, dim, send, bits, np.zeros(send.shape[0], np.int32), 1, seed=17 + b)
    send = np.tile(np.arange(n_rows), 3).astype(np.int32)
    bits = rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=send.shape[0])
    peer = np.sort(rng.integers(0, 2, size=send.shape[0])).astype(np.int32)
    _codec_case(oracle, feat, dim, send, bits, peer, 2, seed=99)


def test_codec_c0(oracle):
    _say("codec c0")
    p = make_partition(CONFIGS["c0"])
    _codec_case(oracle, p.feat, p.cfg.dim, p.send_idx, p.bits, p.peer_of_slot, p.cfg.n_peers, seed=0,
                halo_rows=None)


def test_codec_distributions(oracle):
    """The value distributions of the four workloads at reduced row counts."""
    for name in ("c1", "c2", "c3", "c4"):
        _say(f"codec distribution {name}")
        cfg = replace(CONFIGS[name], n_local=3000, n_halo=2500, n_send=1500, mean_degree=6.0)
        p = make_partition(cfg)
        feat = p.feat if not cfg.backward else np.concatenate([p.feat, p.feat[:1600] * 3], 0)
        send = p.send_idx if not cfg.backward else (p.send_idx % feat.shape[0]).astype(np.int32)
        _codec_case(oracle, np.ascontiguousarray(feat), cfg.dim, send, p.bits, p.peer_of_slot, cfg.n_peers, seed=11)


def test_codec_skips_invalid_slots_and_empty_input(oracle):
    _say("codec invalid slots")
    rng = np.random.default_rng(0)
    dim = 40
    feat = rng.standard_normal((10, dim), dtype=np.float32)
    send = np.array([0, 99, 2, -1, 4], dtype=np.int32)              # 99 and -1 are out of range
    bits = np.array([2, 2, 3, 4, 8], dtype=np.uint8)                # 3 is not a width
    off = np.array([0, 12, 24, 48, 68], dtype=np.int64)
    nbytes = 68 + 40
    got_packed, got_params = _gpu_quantize(feat, dim, send, bits, off, 1, nbytes, fill=0xCD)
    # the oracle rejects invalid slots outright and keys the random stream by position: give it valid
    # stand-ins at the skipped positions and compare only the bytes of the valid slots
    send_v, bits_v = send.copy(), bits.copy()
    send_v[[1, 3]] = 0
    bits_v[2] = 4
    full_packed, full_params, _ = oracle.quantize_pack(feat, dim, send_v, bits_v, off, 1, nbytes)
    assert np.array_equal(got_packed[0:12], full_packed[0:12])
    assert np.array_equal(got_packed[68:108], full_packed[68:108])
    assert np.all(got_packed[12:68] == 0xCD)                          # skipped slots wrote nothing
    assert np.array_equal(got_params[[0, 4]].view(np.uint32), full_params[[0, 4]].view(np.uint32))
    assert np.isnan(got_params[[1, 2, 3]]).all()
    # a row that would overrun the buffer is skipped too
    got_packed, got_params = _gpu_quantize(feat, dim, send[:1], np.array([8], np.uint8), np.array([80], np.int64),
                                           1, 100, fill=0xCD)
    assert np.all(got_packed == 0xCD) and np.isnan(got_params[0]).all()
    # empty input
    e32, e8, e64 = np.zeros(0, np.int32), np.zeros(0, np.uint8), np.zeros(0, np.int64)
    got_packed, _ = _gpu_quantize(feat, dim, e32, e8, e64, 1, 0, fill=0xCD)
    assert np.all(got_packed == 0xCD)


# ------------------------------------------------------------------------------------------------------
# trace for the bit-width assigner (beta of Sec. 4.2)
# ------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("dim,ld", [(128, 128), (602, 608), (602, 602), (300, 320), (7, 7), (5000, 5000)])
def test_quantize_trace_beta(oracle, dim, ld):
    _say(f"beta trace dim={dim} ld={ld}")
    rng = np.random.default_rng(dim)
    n_rows, n = 120, 97
    feat = rng.standard_normal((n_rows, ld), dtype=np.float32) * rng.choice([1e-3, 1.0, 50.0], size=(n_rows, 1)).astype(np.float32)
    feat[2, :dim] = 0.75
    feat[:, dim:] = np.float32(1e30)
    send = rng.integers(0, n_rows, size=n).astype(np.int32)
    send[0] = 2
    bits = np.sort(rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=n))
    perm, off, pbp = oracle.plan_layout(dim, bits, np.zeros(n, np.int32), 1)
    alpha_sq = rng.uniform(0.01, 3.0, size=n).astype(np.float32)
    want_packed, want_params, _ = oracle.quantize_pack(feat, dim, send, bits, off, 9, int(pbp[-1]))
    want_beta = oracle.trace_beta(feat, dim, send, alpha_sq)
    packed = torch.zeros(int(pbp[-1]), dtype=torch.uint8, device=DEV)
    params = torch.zeros((n, 2), dtype=torch.float32, device=DEV)
    beta = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    B.adaqp_quantize_pack_trace(torch.from_numpy(feat).to(DEV), dim, torch.from_numpy(send).to(DEV),
                                torch.from_numpy(bits).to(DEV), torch.from_numpy(off).to(DEV), 9, packed, params,
                                torch.from_numpy(alpha_sq).to(DEV), beta)
    torch.cuda.synchronize()
    assert np.array_equal(packed.cpu().numpy(), want_packed)
    assert np.array_equal(params.cpu().numpy().view(np.uint32), want_params.view(np.uint32))
    assert np.array_equal(beta.cpu().numpy().view(np.uint32), want_beta.view(np.uint32))
    assert want_beta[0] == 0.0
    with pytest.raises(B.AdaqpError):
        B.lib()            # keeps the import used
        B._check(B.lib().adaqp_quantize_pack_trace(1, 1, 8, 8, 1, 1, 1, 1, 0, 1, 8, 1, None, 1, None), "one NULL")


# ------------------------------------------------------------------------------------------------------
# backward receive: de-quantise and add
# ------------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("dim,ld", [(128, 128), (602, 608), (602, 602), (256, 256), (300, 320), (7, 7), (1, 1),
                                    (33, 40), (1100, 1120), (2500, 2500)])
def test_dequant_add(oracle, dim, ld):
    _say(f"dequant add dim={dim} ld={ld}")
    rng = np.random.default_rng(dim + ld)
    n_rows, n = 180, 400
    src = rng.standard_normal((n, dim), dtype=np.float32) * np.float32(1e-3)
    bits = rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=n)
    peer = np.sort(rng.integers(0, 7, size=n)).astype(np.int32)
    perm, off, pbp = oracle.plan_layout(dim, bits, peer, 7)
    s_bits = np.ascontiguousarray(bits[perm])
    packed, params, _ = oracle.quantize_pack(src, dim, perm.astype(np.int32), s_bits, off, 5, int(pbp[-1]))
    dst = rng.integers(60, 160, size=n).astype(np.int32)          # ~4 messages per row, rows 0..59 untouched
    dst[:3] = [-1, n_rows, 61]                                      # two out-of-range destinations: skipped
    order, seg_ptr = B.adaqp_plan_recv_segments(dst)
    grad0 = rng.standard_normal((n_rows, ld), dtype=np.float32)
    want = grad0.copy()
    ok = (dst >= 0) & (dst < n_rows)
    idx = np.nonzero(ok)[0]
    oracle.unpack_dequant_add(packed, params[idx], s_bits[idx], off[idx], dst[idx], dim, want)
    got = torch.from_numpy(grad0).to(DEV)
    B.adaqp_unpack_dequant_add(torch.from_numpy(packed).to(DEV), torch.from_numpy(params).to(DEV),
                               torch.from_numpy(s_bits).to(DEV), torch.from_numpy(off).to(DEV),
                               torch.from_numpy(dst).to(DEV), torch.from_numpy(order).to(DEV),
                               torch.from_numpy(seg_ptr).to(DEV), dim, got)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))


# ------------------------------------------------------------------------------------------------------
# aggregation
# ------------------------------------------------------------------------------------------------------

def _gpu_spmm(rowptr, col, val, rb, re, H, dim, nnz_range=-1, out_fill=7.0, ldo=None):
    n_rows_total = rowptr.shape[0] - 1
    ldo = dim if ldo is None else ldo
    out = torch.full((n_rows_total, ldo), out_fill, dtype=torch.float32, device=DEV)
    nz = int(rowptr[re] - rowptr[rb]) if nnz_range == "exact" else -1
    ws_bytes = B.adaqp_spmm_workspace_bytes(re - rb, nz if nz >= 0 else len(col), dim)
    ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device=DEV)
    colt = torch.from_numpy(col).to(DEV) if len(col) else torch.zeros(1, dtype=torch.int32, device=DEV)[:0]
    valt = torch.from_numpy(val).to(DEV) if len(val) else torch.zeros(1, dtype=torch.float32, device=DEV)[:0]
    B.adaqp_spmm_csr(torch.from_numpy(rowptr).to(DEV), colt, valt, rb, re, torch.from_numpy(H).to(DEV), dim, out,
                     ws, nnz_range=nz)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _check_spmm(oracle, rowptr, col, val, rb, re, H, dim, **kw):
    got = _gpu_spmm(rowptr, col, val, rb, re, H, dim, **kw)
    Hc = np.ascontiguousarray(H[:, :dim]) if H.shape[1] != dim else H
    want, mag = oracle.spmm_csr(rowptr, col, val, rb, re, Hc, dim)
    err = np.abs(got[rb:re, :dim].astype(np.float64) - want)
    tol = SPMM_RTOL * mag + 1e-30
    worst = float((err / tol).max()) if err.size else 0.0
    assert worst <= 1.0, f"worst error {worst:.3f} x tolerance"
    assert np.all(got[:rb] == 7.0) and np.all(got[re:] == 7.0), "rows outside the range were written"
    ldo, ldh = got.shape[1], H.shape[1]
    zero_to = _padded_cols(dim, ldo) if (ldo % 32 == 0 and ldh % 32 == 0) else dim
    assert np.all(got[rb:re, dim:zero_to] == 0.0), "row padding of written rows must be zero"
    assert np.all(got[:, zero_to:] == 7.0), "columns past the padded row were written"
    return got


def _random_graph(rng, n_rows, n_cols, degs):
    rowptr = np.zeros(n_rows + 1, dtype=np.int64)
    cols = []
    for r in range(n_rows):
        d = int(min(degs[r], n_cols))
        c = np.sort(rng.choice(n_cols, size=d, replace=False)) if d else np.zeros(0, np.int64)
        cols.append(c)
        rowptr[r + 1] = rowptr[r] + d
    col = np.concatenate(cols).astype(np.int32) if cols else np.zeros(0, np.int32)
    val = rng.standard_normal(col.shape[0]).astype(np.float32)
    return rowptr, col, val


@pytest.mark.parametrize("dim,ldh", [(128, 128), (602, 602), (256, 256), (300, 300), (1, 1), (7, 9), (66, 66),
                                     (130, 132), (2048, 2048), (2052, 2052), (515, 515),
                                     # line-padded pitches (H padding holds NaN: it must never reach the output)
                                     (602, 608), (300, 320), (7, 32), (250, 256), (2049, 2080), (129, 160)])
def test_spmm_shapes(oracle, dim, ldh):
    _say(f"spmm dim={dim} ldh={ldh}")
    rng = np.random.default_rng(dim)
    n_rows, n_cols = 700, 900
    degs = rng.integers(0, 12, size=n_rows)
    degs[10] = 800                                                     # a row far longer than one piece
    degs[11] = 0
    degs[500:520] = 0                                                  # a run of empty rows
    degs[699] = 300                                                    # heavy last row
    rowptr, col, val = _random_graph(rng, n_rows, n_cols, degs)
    H = np.full((n_cols, ldh), np.nan, dtype=np.float32)
    H[:, :dim] = rng.standard_normal((n_cols, dim), dtype=np.float32)
    ldo = ldh if ldh % 32 == 0 else dim
    _check_spmm(oracle, rowptr, col, val, 0, n_rows, H, dim, ldo=ldo)
    _check_spmm(oracle, rowptr, col, val, 9, 12, H, dim, nnz_range="exact", ldo=ldo)
    _check_spmm(oracle, rowptr, col, val, 495, 700, H, dim, nnz_range="exact", ldo=ldo)
    _check_spmm(oracle, rowptr, col, val, 0, n_rows, H, dim, ldo=dim + 3)            # unpadded output


def test_spmm_degenerate(oracle):
    _say("spmm degenerate")
    rng = np.random.default_rng(1)
    H = rng.standard_normal((5, 16), dtype=np.float32)
    # all rows empty
    rowptr = np.zeros(41, dtype=np.int64)
    got = _check_spmm(oracle, rowptr, np.zeros(0, np.int32), np.zeros(0, np.float32), 0, 40, H, 16)
    assert np.all(got == 0)
    # a single row holding everything
    rowptr = np.array([0, 5], dtype=np.int64)
    _check_spmm(oracle, rowptr, np.arange(5, dtype=np.int32), np.ones(5, np.float32), 0, 1, H, 16)
    # one very long row between empty ones (more entries than any piece)
    n = 5000
    Hbig = rng.standard_normal((n, 64), dtype=np.float32)
    rowptr = np.array([0, 0, 0, n, n, n], dtype=np.int64)
    _check_spmm(oracle, rowptr, np.arange(n, dtype=np.int32), rng.standard_normal(n).astype(np.float32), 0, 5,
                Hbig, 64)
    # out-of-range columns are skipped, not read
    rowptr = np.array([0, 3], dtype=np.int64)
    col = np.array([0, 77, 2], dtype=np.int32)
    val = np.array([1.0, 5.0, 2.0], dtype=np.float32)
    got = _gpu_spmm(rowptr, col, val, 0, 1, H, 16)
    assert np.allclose(got[0], H[0] + 2 * H[2], rtol=1e-6)
    # empty range
    got = _gpu_spmm(np.array([0, 3], dtype=np.int64), col, val, 1, 1, H, 16)
    assert np.all(got == 7.0)


def test_spmm_is_deterministic(oracle):
    _say("spmm determinism")
    p = make_partition(CONFIGS["c0"])
    a = _gpu_spmm(p.rowptr, p.col, p.val, 0, p.n_rows, p.feat, p.cfg.dim)
    b = _gpu_spmm(p.rowptr, p.col, p.val, 0, p.n_rows, p.feat, p.cfg.dim)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_spmm_c0_and_nonnegative_long_rows(oracle):
    _say("spmm c0")
    p = make_partition(CONFIGS["c0"])
    _check_spmm(oracle, p.rowptr, p.col, p.val, 0, p.n_rows, p.feat, p.cfg.dim)
    _check_spmm(oracle, p.rowptr, p.col, p.val, 0, p.n_central, p.feat, p.cfg.dim, nnz_range="exact")
    _check_spmm(oracle, p.rowptr, p.col, p.val, p.n_central, p.n_rows, p.feat, p.cfg.dim, nnz_range="exact")
    # non-negative features and weights: partial sums grow monotonically, the hardest case for fp32 sums
    rng = np.random.default_rng(2)
    n_cols = 30000
    degs = np.array([25000, 3, 12000, 1])
    rowptr, col, val = _random_graph(rng, 4, n_cols, degs)
    val = np.abs(val)
    H = np.abs(rng.standard_normal((n_cols, 256), dtype=np.float32))
    _check_spmm(oracle, rowptr, col, val, 0, 4, H, 256)


# ------------------------------------------------------------------------------------------------------
# aggregation that reads received rows straight from the receive buffer
# ------------------------------------------------------------------------------------------------------

def _packed_case(oracle, rng, n_cols, n_halo, dim, ldh, seed):
    """Received rows for n_halo random columns: (halo, bits, off, packed, params, H_plain, H_ref) where H_plain
    holds NaN in the received rows and H_ref holds what the oracle de-quantises there."""
    halo = np.ascontiguousarray(rng.permutation(n_cols)[:n_halo], dtype=np.int32)
    bits = rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=n_halo)
    peer = np.sort(rng.integers(0, 3, size=n_halo)).astype(np.int32)
    perm, off, pbp = oracle.plan_layout(dim, bits, peer, 3)
    bits = np.ascontiguousarray(bits[perm])
    halo = np.ascontiguousarray(halo[perm])
    src = (rng.standard_normal((n_halo, dim)) * rng.uniform(0.1, 3.0, size=(n_halo, 1))).astype(np.float32)
    packed, params, _ = oracle.quantize_pack(src, dim, np.arange(n_halo, dtype=np.int32), bits, off, seed, int(pbp[-1]))
    H_plain = np.full((n_cols, ldh), np.nan, dtype=np.float32)
    H_plain[:, :dim] = rng.standard_normal((n_cols, dim), dtype=np.float32)
    H_ref = H_plain[:, :dim].copy()
    oracle.unpack_dequant(packed, params, bits, off, halo, dim, H_ref)
    H_plain[halo] = np.nan                                  # the fused path must never read these rows
    return halo, bits, off, packed, params, H_plain, H_ref


def _gpu_spmm_packed(rowptr, col, val, rb, re, H, dim, slot_of_row, packed, params, bits, off, ldo):
    out = torch.full((rowptr.shape[0] - 1, ldo), 7.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(max(B.adaqp_spmm_workspace_bytes(re - rb, len(col), dim), 256), dtype=torch.uint8, device=DEV)
    B.adaqp_spmm_csr_packed(torch.from_numpy(rowptr).to(DEV), torch.from_numpy(col).to(DEV),
                            torch.from_numpy(val).to(DEV), rb, re, torch.from_numpy(H).to(DEV), dim, out,
                            torch.from_numpy(slot_of_row).to(DEV), torch.from_numpy(packed).to(DEV),
                            torch.from_numpy(params).to(DEV), torch.from_numpy(bits).to(DEV),
                            torch.from_numpy(off).to(DEV), ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("dim,ldh", [(128, 128), (602, 608), (602, 602), (300, 300), (7, 7), (1, 1), (66, 66),
                                     (130, 132), (250, 256), (2049, 2080), (2304, 2304), (4100, 4100), (515, 515)])
def test_spmm_packed_rows(oracle, dim, ldh):
    _say(f"spmm from packed rows dim={dim} ldh={ldh}")
    rng = np.random.default_rng(1000 + dim)
    n_rows, n_cols, n_halo = 500, 700, 330
    degs = rng.integers(0, 12, size=n_rows)
    degs[10] = 650                                                     # split over several pieces
    degs[300:310] = 0
    rowptr, col, val = _random_graph(rng, n_rows, n_cols, degs)
    halo, bits, off, packed, params, H_plain, H_ref = _packed_case(oracle, rng, n_cols, n_halo, dim, ldh, seed=77)
    slot_of_row = B.adaqp_plan_slot_of_row(n_cols, halo)
    assert np.array_equal(np.nonzero(slot_of_row >= 0)[0], np.sort(halo))
    assert np.array_equal(halo[slot_of_row[np.sort(halo)]], np.sort(halo))
    ldo = ldh if ldh % 32 == 0 else dim
    got = _gpu_spmm_packed(rowptr, col, val, 0, n_rows, H_plain, dim, slot_of_row, packed, params, bits, off, ldo)
    want, mag = oracle.spmm_csr(rowptr, col, val, 0, n_rows, H_ref, dim)
    err = np.abs(got[:, :dim].astype(np.float64) - want)
    worst = float((err / (SPMM_RTOL * mag + 1e-30)).max())
    assert worst <= 1.0, f"worst error {worst:.3f} x tolerance"
    zero_to = _padded_cols(dim, ldo) if (ldo % 32 == 0 and ldh % 32 == 0) else dim
    assert np.all(got[:, dim:zero_to] == 0.0) and np.all(got[:, zero_to:] == 7.0)
    # bit-identical to de-quantising into H first (same arithmetic, same order)
    H_filled = np.full((n_cols, ldh), np.nan, dtype=np.float32)
    H_filled[:, :dim] = H_ref
    unfused = _gpu_spmm(rowptr, col, val, 0, n_rows, H_filled, dim, ldo=ldo)
    assert np.array_equal(got.view(np.uint32), unfused.view(np.uint32))
    # a sub-range, and a map with unusable slots: those entries read H
    sub = _gpu_spmm_packed(rowptr, col, val, 9, 12, H_plain, dim, slot_of_row, packed, params, bits, off, ldo)
    sub_unfused = _gpu_spmm(rowptr, col, val, 9, 12, H_filled, dim, ldo=ldo)      # same pieces, same order
    assert np.array_equal(sub.view(np.uint32), sub_unfused.view(np.uint32)) and np.all(sub[:9] == 7.0)
    broken = slot_of_row.copy()
    broken[halo[:50]] = n_halo + 5
    H_mixed = H_plain.copy()
    H_mixed[halo[:50], :dim] = H_ref[halo[:50]]
    again = _gpu_spmm_packed(rowptr, col, val, 0, n_rows, H_mixed, dim, broken, packed, params, bits, off, ldo)
    assert np.array_equal(again.view(np.uint32), got.view(np.uint32))


def test_spmm_packed_argument_checks():
    z = torch.zeros(64, dtype=torch.uint8, device=DEV)
    rowptr = torch.zeros(2, dtype=torch.int64, device=DEV)
    col = torch.zeros(1, dtype=torch.int32, device=DEV)[:0]
    val = torch.zeros(1, dtype=torch.float32, device=DEV)[:0]
    H = torch.zeros((4, 32), dtype=torch.float32, device=DEV)
    out = torch.zeros((1, 32), dtype=torch.float32, device=DEV)
    slot = torch.full((4,), -1, dtype=torch.int32, device=DEV)
    ws = torch.empty(4096, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.AdaqpError):                      # a map without slots
        B.adaqp_spmm_csr_packed(rowptr, col, val, 0, 1, H, 32, out, slot, z, torch.zeros((1, 2), device=DEV),
                                z[:0], torch.zeros(1, dtype=torch.int64, device=DEV)[:0], ws)


# ------------------------------------------------------------------------------------------------------
# aggregation tiled over the L2 caches (long rows)
# ------------------------------------------------------------------------------------------------------

def _gpu_spmm_tiled(rowptr, col, val, rb, re, H, dim, ldo, chunk_cols=0):
    n_cols = H.shape[0]
    bounds, off = B.adaqp_plan_spmm_tiles(rowptr, col, rb, re, n_cols)
    out = torch.full((rowptr.shape[0] - 1, ldo), 7.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(max(B.adaqp_spmm_tiled_workspace_bytes(re - rb, dim), 256), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)                                              # NaN patterns: unread unless written first
    B.adaqp_spmm_csr_tiled(torch.from_numpy(rowptr).to(DEV), torch.from_numpy(col).to(DEV),
                           torch.from_numpy(val).to(DEV), rb, re, torch.from_numpy(H).to(DEV), dim, out,
                           torch.from_numpy(off).to(DEV), ws, chunk_cols=chunk_cols)
    torch.cuda.synchronize()
    return out.cpu().numpy(), bounds, off


@pytest.mark.parametrize("dim,ld", [(128, 128), (602, 608), (64, 64), (7, 32), (60, 64), (96, 96), (100, 128),
                                    (130, 160), (256, 256), (2049, 2080)])
def test_spmm_tiled(oracle, dim, ld):
    _say(f"tiled spmm dim={dim} ld={ld}")
    rng = np.random.default_rng(2000 + dim)
    n_rows, n_cols = 300, 900
    degs = rng.integers(0, 150, size=n_rows)
    degs[10] = 880                                                     # nearly every column
    degs[11] = 0
    degs[100:110] = 0
    degs[200:230] = rng.integers(1, 4, size=30)                        # rows that miss most tiles
    rowptr, col, val = _random_graph(rng, n_rows, n_cols, degs)
    H = np.full((n_cols, ld), np.nan, dtype=np.float32)                # NaN in the row padding
    H[:, :dim] = rng.standard_normal((n_cols, dim), dtype=np.float32)
    got, bounds, off = _gpu_spmm_tiled(rowptr, col, val, 0, n_rows, H, dim, ld)
    # the plan: tiles cover the columns, hold about an eighth of the entries each, and count each row's entries
    assert bounds[0] == 0 and bounds[-1] == col.max() + 1 and np.all(np.diff(bounds) >= 0)
    per_tile = np.histogram(col, bins=bounds.astype(np.int64))[0] if False else \
        np.array([np.count_nonzero((col >= bounds[t]) & (col < bounds[t + 1])) for t in range(B.SPMM_TILES)])
    assert per_tile.sum() == len(col) and per_tile.max() <= len(col) / B.SPMM_TILES + degs.max()
    for r in (0, 10, 11, 205, 299):
        c = col[rowptr[r]: rowptr[r + 1]]
        if len(c) >= B.SPMM_TILED_SHORT_ROW:
            assert [int(np.count_nonzero(c < b)) for b in bounds] == off[r].tolist()
        else:                                                          # short rows stay whole, in one tile
            assert off[r].tolist() == [0 if t <= r % B.SPMM_TILES else len(c) for t in range(B.SPMM_TILES + 1)]
    want, mag = oracle.spmm_csr(rowptr, col, val, 0, n_rows, np.ascontiguousarray(H[:, :dim]), dim)
    err = np.abs(got[:, :dim].astype(np.float64) - want)
    worst = float((err / (SPMM_RTOL * mag + 1e-30)).max())
    assert worst <= 1.0, f"worst error {worst:.3f} x tolerance"
    zero_to = _padded_cols(dim, ld)
    assert np.all(got[:, dim:zero_to] == 0.0) and np.all(got[:, zero_to:] == 7.0)
    again, _, _ = _gpu_spmm_tiled(rowptr, col, val, 0, n_rows, H, dim, ld)
    assert np.array_equal(got.view(np.uint32), again.view(np.uint32)), "runs differ"
    assert B.adaqp_spmm_tiled_chunk_cols(bounds, dim) == (64 if dim <= 96 else 128)     # ranges of ~110 columns
    narrow, _, _ = _gpu_spmm_tiled(rowptr, col, val, 0, n_rows, H, dim, ld, chunk_cols=64)
    err = np.abs(narrow[:, :dim].astype(np.float64) - want)
    assert np.all(err <= SPMM_RTOL * mag + 1e-30), "64-column chunks"
    assert np.all(narrow[:, dim:zero_to] == 0.0) and np.all(narrow[:, zero_to:] == 7.0)
    none, _, _ = _gpu_spmm_tiled(rowptr, col, val, 100, 110, H, dim, ld)           # a range of empty rows only
    assert np.all(none[100:110, :zero_to] == 0.0) and np.all(none[:100] == 7.0) and np.all(none[110:] == 7.0)
    sub, _, _ = _gpu_spmm_tiled(rowptr, col, val, 9, 120, H, dim, ld)
    assert np.all(sub[:9] == 7.0) and np.all(sub[120:] == 7.0)
    err = np.abs(sub[9:120, :dim].astype(np.float64) - want[9:120])
    assert np.all(err <= SPMM_RTOL * mag[9:120] + 1e-30)


def test_spmm_tiled_random_shapes(oracle):
    """Seeded sweep over small shapes: fewer columns than tiles, single rows, one dense row, ragged widths."""
    rng = np.random.default_rng(4242)
    dims = [1, 5, 31, 32, 33, 64, 65, 127, 128, 129, 200, 256, 300, 602]
    for case in range(24):
        n_rows = int(rng.choice([1, 2, 3, 15, 16, 17, 100, 257]))
        n_cols = int(rng.choice([1, 2, 7, 8, 9, 70, 500, 1500]))
        dim = int(rng.choice(dims))
        ld = (dim + 31) // 32 * 32
        kind = case % 4
        if kind == 0:
            degs = rng.integers(0, min(n_cols, 200) + 1, size=n_rows)
        elif kind == 1:
            degs = np.full(n_rows, n_cols)                              # dense
        elif kind == 2:
            degs = np.zeros(n_rows, dtype=np.int64)
            degs[rng.integers(0, n_rows)] = n_cols                      # one full row, the rest empty
        else:
            degs = rng.integers(0, 3, size=n_rows)                      # nearly empty
        _say(f"tiled spmm case {case}: rows {n_rows} cols {n_cols} dim {dim} kind {kind}")
        rowptr, col, val = _random_graph(rng, n_rows, n_cols, degs)
        H = np.full((n_cols, ld), np.nan, dtype=np.float32)
        H[:, :dim] = rng.standard_normal((n_cols, dim), dtype=np.float32)
        want, mag = oracle.spmm_csr(rowptr, col, val, 0, n_rows, np.ascontiguousarray(H[:, :dim]), dim)
        for chunk in (0, 64):
            if len(col) == 0:
                # no entries at all: col / val may not even exist; the call only has to zero the rows
                got = torch.full((n_rows, ld), 7.0, dtype=torch.float32, device=DEV)
                off = np.zeros((n_rows, B.SPMM_TILES + 1), dtype=np.int32)
                ws = torch.empty(max(B.adaqp_spmm_tiled_workspace_bytes(n_rows, dim), 256), dtype=torch.uint8,
                                 device=DEV)
                B.adaqp_spmm_csr_tiled(torch.from_numpy(rowptr).to(DEV), torch.zeros(1, dtype=torch.int32, device=DEV)[:0],
                                       torch.zeros(1, dtype=torch.float32, device=DEV)[:0], 0, n_rows,
                                       torch.from_numpy(H).to(DEV), dim, got, torch.from_numpy(off).to(DEV), ws,
                                       chunk_cols=chunk)
                torch.cuda.synchronize()
                got = got.cpu().numpy()
            else:
                got, _, _ = _gpu_spmm_tiled(rowptr, col, val, 0, n_rows, H, dim, ld, chunk_cols=chunk)
            err = np.abs(got[:, :dim].astype(np.float64) - want)
            assert np.all(err <= SPMM_RTOL * mag + 1e-30), f"case {case} chunk {chunk}"
            assert np.all(got[:, dim:] == 0.0), f"case {case}: row padding"


def test_spmm_tiled_rejects_what_it_cannot_do():
    rowptr = np.array([0, 2], dtype=np.int64)
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_spmm_tiles(rowptr, np.array([3, 1], dtype=np.int32), 0, 1, 8)        # not ascending
    with pytest.raises(B.AdaqpError):
        B.adaqp_plan_spmm_tiles(rowptr, np.array([1, 9], dtype=np.int32), 0, 1, 8)        # out of range
    _, off = B.adaqp_plan_spmm_tiles(rowptr, np.array([1, 3], dtype=np.int32), 0, 1, 8)
    H = torch.zeros((8, 30), dtype=torch.float32, device=DEV)                              # pitch not whole lines
    out = torch.zeros((1, 30), dtype=torch.float32, device=DEV)
    ws = torch.empty(4096, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.AdaqpError):
        B.adaqp_spmm_csr_tiled(torch.from_numpy(rowptr).to(DEV), torch.tensor([1, 3], dtype=torch.int32, device=DEV),
                               torch.ones(2, device=DEV), 0, 1, H, 30, out, torch.from_numpy(off).to(DEV), ws)


# ------------------------------------------------------------------------------------------------------
# dense panels of the longest rows on the matrix cores, the tiled kernel for the rest
# ------------------------------------------------------------------------------------------------------

def _gpu_spmm_tiled_and_panels(rowptr, col, val, rb, re, H, dim, ldo, min_row_len, piece_cols, chunk_cols=0):
    n_cols = H.shape[0]
    bounds, off = B.adaqp_plan_spmm_tiles(rowptr, col, rb, re, n_cols)
    plan = B.adaqp_plan_spmm_panels(rowptr, col, val, rb, re, n_cols, bounds, off, min_row_len, piece_cols)
    panels = B.DevicePanels(plan, DEV)
    out = torch.full((rowptr.shape[0] - 1, ldo), 7.0, dtype=torch.float32, device=DEV)
    nbytes = max(B.adaqp_spmm_tiled_workspace_bytes(re - rb, dim),
                 B.adaqp_spmm_panels_workspace_bytes(panels.n_per_tile, dim), 256)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)                                              # NaN patterns: unread unless written first
    Hd = torch.from_numpy(H).to(DEV)
    B.adaqp_spmm_csr_tiled(torch.from_numpy(rowptr).to(DEV), torch.from_numpy(col).to(DEV),
                           torch.from_numpy(val).to(DEV), rb, re, Hd, dim, out, torch.from_numpy(off).to(DEV), ws,
                           chunk_cols=chunk_cols)
    ws.fill_(0xFF)
    B.adaqp_spmm_csr_panels(panels, rb, re, Hd, dim, out, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), plan


@pytest.mark.parametrize("dim,ld", [(128, 128), (602, 608), (64, 64), (7, 32), (100, 128), (130, 160), (256, 256),
                                    (1025, 1056)])
def test_spmm_panels(oracle, dim, ld):
    _say(f"panel spmm dim={dim} ld={ld}")
    rng = np.random.default_rng(3000 + dim)
    n_rows, n_cols = 300, 900
    degs = rng.integers(0, 90, size=n_rows)
    heavy = rng.choice(n_rows, size=70, replace=False)                 # two full panels and a part of a third
    degs[heavy] = rng.integers(100, 600, size=70)
    degs[heavy[0]] = n_cols                                            # every column
    degs[heavy[1]] = 100                                               # exactly the threshold
    rowptr, col, val = _random_graph(rng, n_rows, n_cols, degs)
    H = np.full((n_cols, ld), np.nan, dtype=np.float32)                # NaN in the row padding
    H[:, :dim] = rng.standard_normal((n_cols, dim), dtype=np.float32)
    want, mag = oracle.spmm_csr(rowptr, col, val, 0, n_rows, np.ascontiguousarray(H[:, :dim]), dim)
    zero_to = _padded_cols(dim, ld)
    first = None
    for piece_cols in (8, 64, 1024):
        got, plan = _gpu_spmm_tiled_and_panels(rowptr, col, val, 0, n_rows, H, dim, ld, 100, piece_cols)
        assert plan["n_rows_taken"] == int(np.count_nonzero(degs >= 100)) == 70 and plan["n_panels"] == 3
        err = np.abs(got[:, :dim].astype(np.float64) - want)
        worst = float((err / (SPMM_RTOL * mag + 1e-30)).max())
        assert worst <= 1.0, f"piece_cols {piece_cols}: worst error {worst:.3f} x tolerance"
        assert np.all(got[:, dim:zero_to] == 0.0) and np.all(got[:, zero_to:] == 7.0)
        if first is None:
            first = got
    again, _ = _gpu_spmm_tiled_and_panels(rowptr, col, val, 0, n_rows, H, dim, ld, 100, 8)
    assert np.array_equal(first.view(np.uint32), again.view(np.uint32)), "runs differ"
    # a sub-range: rows outside stay untouched, also those that would be long enough
    sub, plan = _gpu_spmm_tiled_and_panels(rowptr, col, val, 40, 210, H, dim, ld, 100, 64)
    assert plan["n_rows_taken"] == int(np.count_nonzero(degs[40:210] >= 100))
    assert np.all(sub[:40] == 7.0) and np.all(sub[210:] == 7.0)
    err = np.abs(sub[40:210, :dim].astype(np.float64) - want[40:210])
    assert np.all(err <= SPMM_RTOL * mag[40:210] + 1e-30)
    # the panels alone write the rows they list and nothing else
    bounds, off = B.adaqp_plan_spmm_tiles(rowptr, col, 0, n_rows, n_cols)
    plan = B.adaqp_plan_spmm_panels(rowptr, col, val, 0, n_rows, n_cols, bounds, off, 100, 64)
    panels = B.DevicePanels(plan, DEV)
    out = torch.full((n_rows, ld), 7.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(B.adaqp_spmm_panels_workspace_bytes(panels.n_per_tile, dim), dtype=torch.uint8, device=DEV)
    B.adaqp_spmm_csr_panels(panels, 0, n_rows, torch.from_numpy(H).to(DEV), dim, out, ws)
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    listed = np.zeros(n_rows, dtype=bool)
    listed[plan["panel_rows"][plan["panel_rows"] >= 0]] = True
    assert np.all(out[~listed] == 7.0)
    err = np.abs(out[listed, :dim].astype(np.float64) - want[listed])
    assert np.all(err <= SPMM_RTOL * mag[listed] + 1e-30)
    # ... and the tiled kernel leaves exactly those rows alone, so the two may run at the same time: on two
    # streams, a workspace each, the bits are those of one after the other
    rp, cl, vl = (torch.from_numpy(x).to(DEV) for x in (rowptr, col, val))
    Hd, offd = torch.from_numpy(H).to(DEV), torch.from_numpy(off).to(DEV)
    ws_t = torch.empty(B.adaqp_spmm_tiled_workspace_bytes(n_rows, dim), dtype=torch.uint8, device=DEV)
    only_tiled = torch.full((n_rows, ld), 7.0, dtype=torch.float32, device=DEV)
    B.adaqp_spmm_csr_tiled(rp, cl, vl, 0, n_rows, Hd, dim, only_tiled, offd, ws_t)
    torch.cuda.synchronize()
    assert torch.all(only_tiled[torch.from_numpy(listed).to(DEV)] == 7.0)
    one_after_the_other = only_tiled.clone()
    B.adaqp_spmm_csr_panels(panels, 0, n_rows, Hd, dim, one_after_the_other, ws)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)
    together = torch.full((n_rows, ld), 7.0, dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    B.adaqp_spmm_csr_panels(panels, 0, n_rows, Hd, dim, together, ws, stream=s2)
    B.adaqp_spmm_csr_tiled(rp, cl, vl, 0, n_rows, Hd, dim, together, offd, ws_t, stream=s1)
    s1.synchronize()
    s2.synchronize()
    assert torch.equal(together.view(torch.int32), one_after_the_other.view(torch.int32))


def test_non_finite_neighbour_row_and_the_aggregation_paths(oracle):
    """Inputs must be finite.  What happens otherwise is pinned here so that it cannot change unnoticed: an Inf in
    one row of H reaches exactly the rows that have an edge to it in the merge-path and tiled kernels (Sec. 2.1
    Eq. 3 sums over a row's own neighbours); the dense panels multiply every row of H they list by all 32
    coefficients of a panel column, zeros included, so there it reaches every row of the panels that list the
    column (0 * Inf = NaN) - and no row outside them."""
    _say("non-finite row")
    rng = np.random.default_rng(77)
    n_rows, n_cols, dim, ld = 200, 640, 64, 64
    degs = rng.integers(2, 40, size=n_rows)
    heavy = rng.choice(n_rows, size=40, replace=False)
    degs[heavy] = rng.integers(150, 400, size=40)
    rowptr, col, val = _random_graph(rng, n_rows, n_cols, degs)
    H = rng.standard_normal((n_cols, ld), dtype=np.float32)
    bad_col = int(col[rowptr[heavy[0]]])                       # a column that a panel row references
    H[bad_col, 3] = np.inf
    has_edge = np.array([bad_col in col[rowptr[r]: rowptr[r + 1]] for r in range(n_rows)])
    assert has_edge.any() and not has_edge.all()
    merge = _gpu_spmm(rowptr, col, val, 0, n_rows, H, dim)
    tiled, _, _ = _gpu_spmm_tiled(rowptr, col, val, 0, n_rows, H, dim, ld)
    for name, got in (("merge path", merge), ("tiled", tiled)):
        bad_rows = ~np.isfinite(got[:, :dim]).all(axis=1)
        assert np.array_equal(bad_rows, has_edge), name
        assert np.isfinite(got[:, [c for c in range(dim) if c != 3]]).all(), name     # only the column of the Inf
    both, plan = _gpu_spmm_tiled_and_panels(rowptr, col, val, 0, n_rows, H, dim, ld, 150, 64)
    bad_rows = ~np.isfinite(both[:, :dim]).all(axis=1)
    assert np.all(bad_rows[has_edge])                          # never fewer rows than the definition
    panel_rows = plan["panel_rows"].reshape(-1, 32)
    listing = np.zeros(n_rows, dtype=bool)
    for rows in panel_rows:
        rows = rows[rows >= 0]
        if any(bad_col in col[rowptr[r]: rowptr[r + 1]] for r in rows):
            listing[rows] = True
    assert np.array_equal(bad_rows, has_edge | listing)


def test_spmm_panels_random_shapes(oracle):
    """Seeded sweep over small shapes: fewer columns than tiles, a single long row, dense blocks, ragged widths."""
    rng = np.random.default_rng(777)
    dims = [1, 5, 31, 32, 33, 64, 127, 128, 129, 200, 300, 602]
    for case in range(20):
        n_rows = int(rng.choice([1, 2, 31, 32, 33, 65, 150]))
        n_cols = int(rng.choice([1, 3, 7, 8, 9, 70, 500, 1500]))
        dim = int(rng.choice(dims))
        ld = (dim + 31) // 32 * 32
        kind = case % 4
        if kind == 0:
            degs = rng.integers(0, min(n_cols, 300) + 1, size=n_rows)
        elif kind == 1:
            degs = np.full(n_rows, n_cols)                              # dense
        elif kind == 2:
            degs = rng.integers(0, 3, size=n_rows)
            degs[rng.integers(0, n_rows)] = n_cols                      # one full row among nearly empty ones
        else:
            degs = np.where(rng.random(n_rows) < 0.3, n_cols // 2 + 1, 1)
        min_len = int(rng.choice([1, 2, 4, 50]))
        piece_cols = int(rng.choice([8, 16, 256]))
        _say(f"panel spmm case {case}: rows {n_rows} cols {n_cols} dim {dim} kind {kind} min {min_len} piece {piece_cols}")
        rowptr, col, val = _random_graph(rng, n_rows, n_cols, degs)
        if len(col) == 0:
            continue
        H = np.full((n_cols, ld), np.nan, dtype=np.float32)
        H[:, :dim] = rng.standard_normal((n_cols, dim), dtype=np.float32)
        want, mag = oracle.spmm_csr(rowptr, col, val, 0, n_rows, np.ascontiguousarray(H[:, :dim]), dim)
        got, plan = _gpu_spmm_tiled_and_panels(rowptr, col, val, 0, n_rows, H, dim, ld, min_len, piece_cols)
        assert (plan is None) == (not np.any(np.diff(rowptr) >= min_len))
        err = np.abs(got[:, :dim].astype(np.float64) - want)
        assert np.all(err <= SPMM_RTOL * mag + 1e-30), f"case {case}"
        assert np.all(got[:, dim:] == 0.0), f"case {case}: row padding"


def test_spmm_panels_rejects_what_it_cannot_do():
    rng = np.random.default_rng(5)
    rowptr, col, val = _random_graph(rng, 40, 64, np.full(40, 20))
    bounds, off = B.adaqp_plan_spmm_tiles(rowptr, col, 0, 40, 64)
    panels = B.DevicePanels(B.adaqp_plan_spmm_panels(rowptr, col, val, 0, 40, 64, bounds, off, 10, 16), DEV)
    assert panels and panels.c.n_panels == 2
    need = B.adaqp_spmm_panels_workspace_bytes(panels.n_per_tile, 32)
    H = torch.zeros((64, 32), dtype=torch.float32, device=DEV)
    out = torch.zeros((40, 32), dtype=torch.float32, device=DEV)
    with pytest.raises(B.AdaqpError):                                      # workspace too small
        B.adaqp_spmm_csr_panels(panels, 0, 40, H, 32, out, torch.empty(need - 256, dtype=torch.uint8, device=DEV))
    Hbad = torch.zeros((64, 40), dtype=torch.float32, device=DEV)         # pitch not whole lines
    with pytest.raises(B.AdaqpError):
        B.adaqp_spmm_csr_panels(panels, 0, 40, Hbad, 32, out, torch.empty(need, dtype=torch.uint8, device=DEV))
    empty = B.DevicePanels(None)                                           # no panels: a successful no-op
    B.adaqp_spmm_csr_panels(empty, 0, 40, H, 32, out, torch.empty(256, dtype=torch.uint8, device=DEV))
    torch.cuda.synchronize()
    assert torch.all(out == 0)


# ------------------------------------------------------------------------------------------------------
# the layer step
# ------------------------------------------------------------------------------------------------------

def _oracle_layer(oracle, p, seed):
    """Composes the oracle's pieces in the order of Sec. 3.1: quantise, exchange (identity), de-quantise,
    aggregate.  Returns (packed, params, feat_after, out64, mag64)."""
    cfg = p.cfg
    perm, off, pbp = oracle.plan_layout(cfg.dim, p.bits, p.peer_of_slot, cfg.n_peers)
    s_idx = np.ascontiguousarray(p.send_idx[perm])
    s_bits = np.ascontiguousarray(p.bits[perm])
    if not cfg.backward:
        packed, params, _ = oracle.quantize_pack(p.feat, cfg.dim, s_idx, s_bits, off, seed, int(pbp[-1]))
        feat = p.feat.copy()
        oracle.unpack_dequant(packed, params, s_bits, off, np.ascontiguousarray(p.halo_idx[perm]), cfg.dim, feat)
        out64, mag = oracle.spmm_csr(p.rowptr, p.col, p.val, 0, p.n_rows, feat, cfg.dim)
        return packed, params, feat, out64, mag
    out = np.zeros((p.n_rows, cfg.dim), dtype=np.float32)
    out64, mag = oracle.spmm_csr(p.rowptr, p.col, p.val, 0, p.n_rows, p.feat, cfg.dim, out=out)
    return None, None, None, out64, mag


@pytest.mark.parametrize("name", ["c0", "c0_backward"])
def test_layer_step_matches_oracle_in_every_schedule(oracle, name):
    _say(f"layer step {name}")
    if name == "c0":
        p = make_partition(CONFIGS["c0"])
    else:
        p = make_partition(replace(CONFIGS["c4"], n_local=2000, n_halo=1800, n_send=1500, mean_degree=9.0, dim=128))
    cfg = p.cfg
    seed = 1234
    packed_w, params_w, feat_w, out64, mag = _oracle_layer(oracle, p, seed)
    results = []
    for schedule in (B.SERIAL, B.ISOLATED, B.FREE):
        L = LayerStep(p, DEV, seed=seed, backward_receive=False)
        if not cfg.backward:
            # poison what the step must produce, so that a missing dependency shows as NaN
            L.feat[cfg.n_local: cfg.n_local + cfg.n_send] = float("nan")
        L.out.fill_(float("nan"))
        torch.cuda.synchronize()
        L.run(schedule)
        L.synchronize()
        out = L.out.cpu().numpy()
        err = np.abs(out.astype(np.float64) - out64)
        assert np.all(err <= SPMM_RTOL * mag + 1e-30), f"schedule {schedule}: aggregation off"
        packed = L.recv_packed.cpu().numpy()[: L.plan.packed_bytes]
        params = L.recv_params.cpu().numpy()[: L.plan.n]
        if not cfg.backward:
            want_beta = oracle.trace_beta(p.feat, cfg.dim, L.plan.send_idx_host, L.alpha_sq_host)
            assert np.array_equal(L.beta.cpu().numpy().view(np.uint32), want_beta.view(np.uint32))
            assert np.array_equal(packed, packed_w)
            assert np.array_equal(params.view(np.uint32), params_w.view(np.uint32))
            assert np.array_equal(L.feat.cpu().numpy().view(np.uint32), feat_w.view(np.uint32))
        results.append((out, packed, params))
    for out, packed, params in results[1:]:
        assert np.array_equal(out.view(np.uint32), results[0][0].view(np.uint32)), "schedules disagree"
        assert np.array_equal(packed, results[0][1]) and np.array_equal(params.view(np.uint32),
                                                                        results[0][2].view(np.uint32))
    if cfg.backward:
        # the oracle quantises the GPU's own fp32 aggregate: the codes depend on every bit of the input, and
        # the aggregate is only specified to a tolerance
        L = LayerStep(p, DEV, seed=seed, backward_receive=False)
        L.run(B.SERIAL)
        L.synchronize()
        g = L.out.cpu().numpy()
        want_packed, want_params, _ = oracle.quantize_pack(g, cfg.dim, L.plan.send_idx_host, L.plan.bits_host,
                                                           L.plan.row_offset_host, seed, L.plan.packed_bytes)
        assert np.array_equal(L.recv_packed.cpu().numpy()[: L.plan.packed_bytes], want_packed)
        assert np.array_equal(L.recv_params.cpu().numpy()[: L.plan.n].view(np.uint32), want_params.view(np.uint32))
        # with the receive side switched on, the received gradients are added to the local rows in slot order:
        # the oracle adds the same received bytes to the aggregate computed above
        want_out = np.ascontiguousarray(g.copy())
        oracle.unpack_dequant_add(want_packed, want_params, L.plan.bits_host, L.plan.row_offset_host,
                                  L.plan.halo_idx_host, cfg.dim, want_out)
        assert not np.array_equal(want_out, g)
        for schedule in (B.SERIAL, B.ISOLATED, B.FREE):
            L2 = LayerStep(p, DEV, seed=seed)
            L2.out.fill_(float("nan"))
            L2.run(schedule)
            L2.synchronize()
            assert np.array_equal(L2.out.cpu().numpy().view(np.uint32), want_out.view(np.uint32)), \
                f"schedule {schedule}: backward receive differs"


def test_layer_step_fused_receive(oracle):
    """Forward step whose dependent aggregation reads the receive buffer: same output bits as the step that
    de-quantises into the feature matrix first, and the halo rows of the feature matrix stay untouched."""
    p = make_partition(CONFIGS["c0"])
    cfg = p.cfg
    seed = 1234
    _, _, _, out64, mag = _oracle_layer(oracle, p, seed)
    plain = LayerStep(p, DEV, seed=seed)
    plain.run(B.SERIAL)
    plain.synchronize()
    want = plain.out.cpu().numpy()
    for schedule in (B.SERIAL, B.ISOLATED, B.FREE):
        L = LayerStep(p, DEV, seed=seed, fused_receive=True)
        L.feat[cfg.n_local: cfg.n_local + cfg.n_send] = float("nan")
        L.out.fill_(float("nan"))
        torch.cuda.synchronize()
        L.run(schedule)
        L.synchronize()
        out = L.out.cpu().numpy()
        assert np.all(np.abs(out.astype(np.float64) - out64) <= SPMM_RTOL * mag + 1e-30)
        assert np.array_equal(out.view(np.uint32), want.view(np.uint32)), f"schedule {schedule}"
        assert bool(torch.isnan(L.feat[cfg.n_local: cfg.n_local + cfg.n_send]).all())
        assert np.array_equal(L.recv_packed.cpu().numpy(), plain.recv_packed.cpu().numpy())


def test_mean_aggregator_layer_step(oracle):
    """GraphSAGE-style mean coefficients (1 / row degree) through the same step."""
    p = make_partition(replace(CONFIGS["c0"], aggregator="mean"))
    _, _, feat_w, out64, mag = _oracle_layer(oracle, p, 9)
    L = LayerStep(p, DEV, seed=9)
    L.out.fill_(float("nan"))
    L.run(B.ISOLATED)
    L.synchronize()
    out = L.out.cpu().numpy()
    assert np.all(np.abs(out.astype(np.float64) - out64) <= SPMM_RTOL * mag + 1e-30)
    assert np.array_equal(L.feat.cpu().numpy().view(np.uint32), feat_w.view(np.uint32))
    # a mean of values stays inside their range
    lo, hi = feat_w.min(), feat_w.max()
    assert out.min() >= lo - 1e-4 and out.max() <= hi + 1e-4


def test_trace_assign_replan_loop(oracle):
    """One period of Sec. 3.3: the step traces beta, the assigner turns it into widths, the next step runs with
    the new layout.  The oracle does the same from its own trace; widths and bytes must agree exactly."""
    import dataclasses
    from oracle import assigner as A
    p = make_partition(CONFIGS["c0"])
    cfg = p.cfg
    seed = 77
    L = LayerStep(p, DEV, seed=seed)
    L.run(B.SERIAL)
    L.synchronize()
    pl = L.plan
    beta_gpu = L.beta.cpu().numpy()
    peer_sorted = np.ascontiguousarray(p.peer_of_slot[pl.perm])
    theta = np.array([1.0, 1.5, 0.7]) * 1e-8
    gamma = np.full(cfg.n_peers, 1e-5)
    lam, group = 1e-7, 20
    bits_sorted, obj = B.adaqp_assign_bits(beta_gpu, peer_sorted, cfg.n_peers, cfg.dim, group, lam, theta, gamma)
    beta_cpu = oracle.trace_beta(p.feat, cfg.dim, pl.send_idx_host, L.alpha_sq_host)
    want_bits = A.greedy(beta_cpu, peer_sorted, cfg.n_peers, cfg.dim, group, lam, theta, gamma)
    assert np.array_equal(bits_sorted, want_bits)
    assert set(np.unique(bits_sorted)) == {2, 4, 8}
    f, _, _ = A.objective(beta_cpu, peer_sorted, cfg.n_peers, cfg.dim, bits_sorted, lam, theta, gamma)
    assert obj[0] == pytest.approx(f, rel=1e-12)
    # the assignment beats the one it replaces on the objective it was chosen for
    f_old, _, _ = A.objective(beta_cpu, peer_sorted, cfg.n_peers, cfg.dim, pl.bits_host, lam, theta, gamma)
    assert f < f_old
    bits_new = np.zeros_like(p.bits)
    bits_new[pl.perm] = bits_sorted                                  # back to the caller's slot order
    p2 = dataclasses.replace(p, bits=bits_new)
    packed_w, params_w, feat_w, out64, mag = _oracle_layer(oracle, p2, seed)
    L2 = LayerStep(p2, DEV, seed=seed)
    L2.run(B.ISOLATED)
    L2.synchronize()
    assert np.array_equal(L2.recv_packed.cpu().numpy()[: L2.plan.packed_bytes], packed_w)
    assert np.array_equal(L2.feat.cpu().numpy().view(np.uint32), feat_w.view(np.uint32))
    assert np.all(np.abs(L2.out.cpu().numpy().astype(np.float64) - out64) <= SPMM_RTOL * mag + 1e-30)


@pytest.mark.parametrize("name", ["c0", "c0_backward"])
def test_layer_step_with_tiled_aggregation(oracle, name):
    """Both row ranges through the L2-tiled kernel, every schedule, forward and backward."""
    if name == "c0":
        p = make_partition(CONFIGS["c0"])
    else:
        p = make_partition(replace(CONFIGS["c4"], n_local=2000, n_halo=1800, n_send=1500, mean_degree=9.0, dim=128))
    cfg = p.cfg
    seed = 4321
    packed_w, params_w, feat_w, out64, mag = _oracle_layer(oracle, p, seed)
    first = None
    for schedule in (B.SERIAL, B.ISOLATED, B.FREE):
        L = LayerStep(p, DEV, seed=seed, tiled=True, backward_receive=False)
        assert L.tile_off_overlap is not None and L.tile_off_dependent is not None
        if not cfg.backward:
            L.feat[cfg.n_local: cfg.n_local + cfg.n_send] = float("nan")
        L.out.fill_(float("nan"))
        torch.cuda.synchronize()
        L.run(schedule)
        L.synchronize()
        out = L.out.cpu().numpy()
        assert np.all(np.abs(out.astype(np.float64) - out64) <= SPMM_RTOL * mag + 1e-30), f"schedule {schedule}"
        if not cfg.backward:
            assert np.array_equal(L.recv_packed.cpu().numpy()[: L.plan.packed_bytes], packed_w)
            assert np.array_equal(L.feat.cpu().numpy().view(np.uint32), feat_w.view(np.uint32))
        if first is None:
            first = out
        assert np.array_equal(out.view(np.uint32), first.view(np.uint32)), "schedules disagree"


@pytest.mark.parametrize("name", ["c0", "c0_backward"])
def test_layer_step_with_panels(oracle, name):
    """Tiled aggregation with the longer rows of both ranges in dense panels, every schedule, both directions."""
    if name == "c0":
        p = make_partition(CONFIGS["c0"])
    else:
        p = make_partition(replace(CONFIGS["c4"], n_local=2000, n_halo=1800, n_send=1500, mean_degree=9.0, dim=128))
    cfg = p.cfg
    seed = 8765
    deg = np.diff(p.rowptr)
    min_row = max(int(np.quantile(deg[deg > 0], 0.9)), 2)               # the longest tenth of the rows
    packed_w, params_w, feat_w, out64, mag = _oracle_layer(oracle, p, seed)
    first = None
    for schedule in (B.SERIAL, B.ISOLATED, B.FREE):
        L = LayerStep(p, DEV, seed=seed, tiled=True, panels=True, backward_receive=False, panel_min_row=min_row)
        assert L.panels_overlap and L.panels_dependent
        n_taken = int(np.count_nonzero(L.panels_overlap.tensors["panel_rows"].cpu().numpy() >= 0)) + \
            int(np.count_nonzero(L.panels_dependent.tensors["panel_rows"].cpu().numpy() >= 0))
        ob, oe = p.overlap_rows
        db, de = p.dependent_rows
        assert n_taken == int(np.count_nonzero(deg[ob:oe] >= min_row)) + int(np.count_nonzero(deg[db:de] >= min_row))
        if not cfg.backward:
            L.feat[cfg.n_local: cfg.n_local + cfg.n_send] = float("nan")
        L.out.fill_(float("nan"))
        torch.cuda.synchronize()
        L.run(schedule)
        L.synchronize()
        out = L.out.cpu().numpy()
        assert np.all(np.abs(out.astype(np.float64) - out64) <= SPMM_RTOL * mag + 1e-30), f"schedule {schedule}"
        if not cfg.backward:
            assert np.array_equal(L.recv_packed.cpu().numpy()[: L.plan.packed_bytes], packed_w)
            assert np.array_equal(L.feat.cpu().numpy().view(np.uint32), feat_w.view(np.uint32))
        if first is None:
            first = out
        assert np.array_equal(out.view(np.uint32), first.view(np.uint32)), "schedules disagree"
    # without panels the same rows come out of the tiled kernel: same sums up to rounding order
    L = LayerStep(p, DEV, seed=seed, tiled=True, backward_receive=False, panels=False)
    assert not L.panels_overlap and not L.panels_dependent
    L.run(B.SERIAL)
    L.synchronize()
    assert np.all(np.abs(L.out.cpu().numpy().astype(np.float64) - out64) <= SPMM_RTOL * mag + 1e-30)


@pytest.mark.parametrize("schedule_name", ["serial", "isolated", "isolated_tiled_panels", "free_tiled_panels"])
def test_layer_step_captured_in_a_graph(schedule_name):
    """The step allocates nothing and clears nothing with memset, so it can be captured into a HIP graph; every
    replay (with eager work and synchronisations in between) must give the bits of the eager step.  With tiles
    and panels in both row ranges the two streams wait for each other twice more (the panel kernels run beside
    the tiled ones)."""
    schedule = {"serial": B.SERIAL, "isolated": B.ISOLATED, "free": B.FREE}[schedule_name.split("_")[0]]
    p = make_partition(CONFIGS["c0"])
    cfg = p.cfg
    if schedule_name.endswith("tiled_panels"):
        deg = np.diff(p.rowptr)
        L = LayerStep(p, DEV, seed=99, tiled=True, panels=True,
                      panel_min_row=max(int(np.quantile(deg[deg > 0], 0.9)), 2))
        assert L.panels_overlap and L.panels_dependent
    else:
        L = LayerStep(p, DEV, seed=99)
    L.run(schedule)
    L.synchronize()
    want_out = L.out.clone()
    want_feat = L.feat.clone()
    want_packed = L.recv_packed.clone()
    desc = L.desc(schedule)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=L.stream_msg):
        B.adaqp_layer_step(desc)
    for replay in range(3):
        L.out.fill_(float("nan"))                                   # eager work between the replays
        L.feat[cfg.n_local: cfg.n_local + cfg.n_send] = float("nan")
        L.recv_packed.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(L.recv_packed, want_packed), f"replay {replay}: packed bytes"
        assert torch.equal(L.feat.view(torch.int32), want_feat.view(torch.int32)), f"replay {replay}: halo rows"
        assert torch.equal(L.out.view(torch.int32), want_out.view(torch.int32)), f"replay {replay}: aggregate"
