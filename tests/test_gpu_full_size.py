"""GPU parity at the full workload sizes, in the launch configuration bench.py times (line-padded matrices,
one adaqp_layer_step): sampled slots and rows are recomputed one by one by the CPU oracle, plus properties
that hold at any size."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2306_01381_amd import binding as B                      # noqa: E402
from paper_2306_01381_amd.layer import LayerStep                    # noqa: E402
from paper_2306_01381_amd.synth import CONFIGS, make_partition      # noqa: E402

SPMM_RTOL = 1e-5
SEED = 2306


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.lib()


def _sample_slots(rng, plan, k):
    n = plan.n
    picks = set(rng.integers(0, n, size=k).tolist()) | {0, n - 1}
    change = np.nonzero(np.diff(plan.bits_host.astype(np.int32)) != 0)[0]        # width-group boundaries
    for c in change[:40]:
        picks |= {int(c), int(c) + 1}
    return sorted(picks)


def _sample_rows(rng, rowptr, lo, hi, k):
    deg = np.diff(rowptr[lo: hi + 1])
    picks = set((lo + rng.integers(0, hi - lo, size=k)).tolist()) | {lo, hi - 1}
    picks |= set((lo + np.argsort(deg)[-4:]).tolist())        # the longest rows (split over many pieces)
    picks |= set((lo + np.argsort(deg)[:2]).tolist())         # the shortest
    # rows on both sides of the length from which a row is aggregated in a dense panel, and a few inside panels
    order = np.argsort(-deg, kind="stable")
    n_long = int(np.count_nonzero(deg >= B.SPMM_PANEL_MIN_ROW))
    if n_long:
        picks |= set((lo + order[max(n_long - 3, 0): n_long + 3]).tolist())
        picks |= set((lo + order[rng.integers(0, n_long, size=6)]).tolist())
        picks |= set((lo + order[[31, 32, 33]][: max(min(n_long - 31, 3), 0)]).tolist())     # around a panel seam
    return sorted(picks)


def _check_rows(oracle, p, H_host, out, rows, dim):
    worst = 0.0
    for r in rows:
        want, mag = oracle.spmm_csr(p.rowptr, p.col, p.val, r, r + 1, H_host, dim)
        err = np.abs(out[r].astype(np.float64) - want[0])
        worst = max(worst, float((err / (SPMM_RTOL * mag[0] + 1e-30)).max()))
    assert worst <= 1.0, f"worst aggregation error {worst:.3f} x tolerance"
    return worst


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
def test_full_size_layer_step(oracle, name):
    cfg = CONFIGS[name]
    _say(f"full size {name}: generating")
    p = make_partition(cfg)
    dim = cfg.dim
    L = LayerStep(p, "cuda:0", seed=SEED, backward_receive=False)
    if not cfg.backward:
        L.feat[cfg.n_local: cfg.n_local + cfg.n_send] = float("nan")     # must be produced by the step
    L.out.fill_(float("nan"))
    torch.cuda.synchronize()
    _say(f"full size {name}: layer step")
    L.run(B.SERIAL)
    L.synchronize()
    pl = L.plan
    rng = np.random.default_rng(99)

    out = L.out.cpu().numpy()
    packed = L.recv_packed.cpu().numpy()[: pl.packed_bytes]
    params = L.recv_params.cpu().numpy()[: pl.n]
    assert np.isfinite(out).all() and np.isfinite(params).all()
    assert np.all(params[:, 1] >= 0)
    assert np.array_equal(L.packed.cpu().numpy()[: pl.packed_bytes], packed)      # the loop-back copy

    # ---- aggregation: sampled rows of both launches ----
    H_host = np.ascontiguousarray(L.feat.cpu().numpy())       # forward: after de-quantisation
    rows = _sample_rows(rng, p.rowptr, *p.overlap_rows, 60) + _sample_rows(rng, p.rowptr, *p.dependent_rows, 60)
    worst = _check_rows(oracle, p, H_host, out, rows, dim)
    _say(f"full size {name}: {len(rows)} rows ok, worst {worst:.3f} of tolerance")

    # ---- send side: sampled slots, recomputed alone (the random stream is keyed by the slot number) ----
    src = out if cfg.backward else p.feat                     # backward quantises the GPU's own aggregate
    src = np.ascontiguousarray(src)
    slots = _sample_slots(rng, pl, 250)
    for s in slots:
        b = int(pl.bits_host[s])
        stride = B.adaqp_row_stride(dim, b)
        want_row, want_par, _ = oracle.quantize_pack(src, dim, pl.send_idx_host[s: s + 1], pl.bits_host[s: s + 1],
                                                     np.zeros(1, np.int64), SEED, stride, slot_base=s)
        off = int(pl.row_offset_host[s])
        assert np.array_equal(packed[off: off + stride], want_row), f"slot {s}: packed bytes differ"
        assert np.array_equal(params[s].view(np.uint32), want_par[0].view(np.uint32)), f"slot {s}: (Z,S) differ"
    _say(f"full size {name}: {len(slots)} slots ok")

    # ---- receive side: the same slots, de-quantised alone ----
    if not cfg.backward:
        feat_after = H_host
        for s in slots:
            b = int(pl.bits_host[s])
            stride = B.adaqp_row_stride(dim, b)
            off = int(pl.row_offset_host[s])
            one = np.zeros((1, dim), dtype=np.float32)
            oracle.unpack_dequant(packed[off: off + stride], params[s: s + 1], pl.bits_host[s: s + 1],
                                  np.zeros(1, np.int64), np.zeros(1, np.int32), dim, one)
            assert np.array_equal(feat_after[pl.halo_idx_host[s]].view(np.uint32), one[0].view(np.uint32)), \
                f"slot {s}: de-quantised row differs"
        # rows that are not received keep their contents; local rows are never touched
        assert np.array_equal(feat_after[: cfg.n_local].view(np.uint32), p.feat[: cfg.n_local].view(np.uint32))
        untouched = np.ones(p.n_cols, dtype=bool)
        untouched[pl.halo_idx_host] = False
        untouched[: cfg.n_local] = False
        assert np.array_equal(feat_after[untouched].view(np.uint32), p.feat[untouched].view(np.uint32))
        # every received row lies within one quantisation step of what was sent (Eq. 4-5)
        sent = p.feat[pl.send_idx_host]
        got = feat_after[pl.halo_idx_host]
        assert np.all(np.abs(got - sent) <= params[:, 1:2] * (1 + 1e-4) + 1e-30)

    # ---- the two-stream schedules (bench.py times `isolated` where the step pairs a panel kernel with a tiled
    # ---- one): the same bits as the serial step checked above ----
    want_out, want_feat = L.out.clone(), L.feat.clone()
    for schedule in (B.ISOLATED, B.FREE):
        if not cfg.backward:
            L.feat[cfg.n_local: cfg.n_local + cfg.n_send] = float("nan")
        L.out.fill_(float("nan"))
        L.recv_packed.zero_()
        torch.cuda.synchronize()
        L.run(schedule)
        L.synchronize()
        assert torch.equal(L.out.view(torch.int32), want_out.view(torch.int32)), f"schedule {schedule}: aggregate"
        assert torch.equal(L.feat.view(torch.int32), want_feat.view(torch.int32)), f"schedule {schedule}: halo rows"
        assert np.array_equal(L.recv_packed.cpu().numpy()[: pl.packed_bytes], packed), f"schedule {schedule}: bytes"
    _say(f"full size {name}: isolated and free schedules give the serial step's bits")


def test_full_size_backward_receive(oracle):
    """c4 with the receive side on: the received gradients are added to the local rows in slot order."""
    cfg = CONFIGS["c4"]
    _say("full size c4 backward receive: generating")
    p = make_partition(cfg)
    dim = cfg.dim
    base = LayerStep(p, "cuda:0", seed=SEED, backward_receive=False)
    base.run(B.SERIAL)
    base.synchronize()
    out0 = base.out.cpu().numpy()
    packed = base.recv_packed.cpu().numpy()[: base.plan.packed_bytes]
    params = base.recv_params.cpu().numpy()[: base.plan.n]
    del base
    L = LayerStep(p, "cuda:0", seed=SEED)
    L.out.fill_(float("nan"))
    L.run(B.ISOLATED)
    L.synchronize()
    out1 = L.out.cpu().numpy()
    pl = L.plan
    assert np.array_equal(L.recv_packed.cpu().numpy()[: pl.packed_bytes], packed)
    dst = pl.halo_idx_host
    touched = np.zeros(p.n_rows, dtype=bool)
    touched[dst] = True
    assert np.array_equal(out1[~touched].view(np.uint32), out0[~touched].view(np.uint32))
    rng = np.random.default_rng(5)
    counts = np.bincount(dst, minlength=p.n_rows)
    rows = set(rng.choice(np.nonzero(touched)[0], size=200, replace=False).tolist())
    rows |= set(np.argsort(counts)[-5:].tolist())                     # the rows that hear from the most peers
    for r in sorted(rows):
        slots = np.nonzero(dst == r)[0]                                # ascending = slot order
        want = np.ascontiguousarray(out0[r: r + 1].copy())
        for s in slots:
            b = int(pl.bits_host[s])
            stride = B.adaqp_row_stride(dim, b)
            off = int(pl.row_offset_host[s])
            oracle.unpack_dequant_add(packed[off: off + stride], params[s: s + 1], pl.bits_host[s: s + 1],
                                      np.zeros(1, np.int64), np.zeros(1, np.int32), dim, want)
        assert np.array_equal(out1[r].view(np.uint32), want[0].view(np.uint32)), f"row {r}: {len(slots)} messages"
    _say(f"full size c4 backward receive: {len(rows)} rows ok, up to {counts.max()} messages per row")


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_full_size_fused_receive(oracle, name):
    """The step whose marginal aggregation reads the receive buffer directly: the halo rows of the feature
    matrix are never written, the output has the bits of the plain step, and sampled marginal rows agree
    with the oracle run on the oracle's own de-quantised rows."""
    cfg = CONFIGS[name]
    _say(f"full size {name} fused receive: generating")
    p = make_partition(cfg)
    dim = cfg.dim
    L = LayerStep(p, "cuda:0", seed=SEED, tiled=False)       # same kernel, same summation order in both runs
    L.run(B.SERIAL)
    L.synchronize()
    plain = L.out.cpu().numpy()
    L.set_fused_receive(True)
    L.feat[cfg.n_local: cfg.n_local + cfg.n_send] = float("nan")
    L.out.fill_(float("nan"))
    torch.cuda.synchronize()
    _say(f"full size {name} fused receive: layer step")
    L.run(B.ISOLATED)
    L.synchronize()
    out = L.out.cpu().numpy()
    assert np.array_equal(out.view(np.uint32), plain.view(np.uint32))
    assert bool(torch.isnan(L.feat[cfg.n_local: cfg.n_local + cfg.n_send]).all())
    pl = L.plan
    packed = L.recv_packed.cpu().numpy()[: pl.packed_bytes]
    params = L.recv_params.cpu().numpy()[: pl.n]
    H = p.feat.copy()
    oracle.unpack_dequant(packed, params, pl.bits_host, pl.row_offset_host, pl.halo_idx_host, dim, H)
    rng = np.random.default_rng(3)
    rows = _sample_rows(rng, p.rowptr, *p.dependent_rows, 60)
    worst = _check_rows(oracle, p, H, out, rows, dim)
    _say(f"full size {name} fused receive: {len(rows)} rows ok, worst {worst:.3f} of tolerance")
