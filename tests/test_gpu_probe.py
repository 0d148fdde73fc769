"""The measurement aids of include/adaqp_probe.h: they stay inside the stated extents, and the workgroup -> XCD
mapping that the tiled and panel aggregation kernels are scheduled around is what this GPU does."""
import sys

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2306_01381_amd import binding as B                      # noqa: E402

DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.lib()


def test_consecutive_workgroups_land_on_consecutive_xcds():
    """adaqp_spmm_csr_tiled / _panels give workgroup i the column range i mod 8: that keeps one range per L2 only
    if a grid's workgroups are dealt to the eight XCDs in turn."""
    _say("xcd map")
    for n in (8, 64, 1000, 4096):
        xcd = B.adaqp_probe_xcd_of_workgroup(n, DEV)
        torch.cuda.synchronize()
        x = xcd.cpu().numpy()
        assert x.min() >= 0 and x.max() < B.SPMM_TILES
        assert np.array_equal((x - x[0]) % B.SPMM_TILES, np.arange(n) % B.SPMM_TILES), \
            "workgroups are not dealt to the XCDs round-robin: the tiled aggregation would lose its L2 locality"
        assert len(set(x[: B.SPMM_TILES].tolist())) == B.SPMM_TILES


@pytest.mark.parametrize("dim,ld", [(602, 608), (256, 256), (300, 320), (128, 128)])
def test_no_compute_twin_writes_only_what_the_kernel_writes(dim, ld):
    _say(f"probe twin dim={dim}")
    rng = np.random.default_rng(dim)
    n_rows, n = 500, 333
    feat = torch.from_numpy(rng.standard_normal((n_rows, ld), dtype=np.float32)).to(DEV)
    bits = rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=n)
    peer = np.sort(rng.integers(0, 3, size=n)).astype(np.int32)
    perm, off, pbp = B.adaqp_plan_layout(dim, bits, peer, 3)
    send = rng.integers(0, n_rows, size=n).astype(np.int32)[perm]
    nbytes = int(pbp[-1])
    guard = 4096
    packed = torch.full((nbytes + guard,), 0xAB, dtype=torch.uint8, device=DEV)
    params = torch.full((n + 8, 2), 5.0, dtype=torch.float32, device=DEV)
    B.adaqp_probe_quantize_pack(feat[:, :dim] if ld != dim else feat, dim, torch.from_numpy(send).to(DEV),
                                torch.from_numpy(np.ascontiguousarray(bits[perm])).to(DEV),
                                torch.from_numpy(off).to(DEV), packed[:nbytes], params[:n])
    torch.cuda.synchronize()
    assert bool((packed[nbytes:] == 0xAB).all()) and bool((params[n:] == 5.0).all())
    assert not bool((params[:n] == 5.0).all())


def test_stream_probe_stays_inside_its_buffers():
    _say("probe stream")
    nbytes = 3_000_016
    big = torch.zeros(nbytes + 4096, dtype=torch.uint8, device=DEV)
    small = torch.zeros(nbytes // 8 + 4096 + 4096, dtype=torch.uint8, device=DEV)
    big[:nbytes] = 1
    small[nbytes // 8 + 4096:] = 0x5A
    B.adaqp_probe_stream(big, small[: nbytes // 8 + 4096], nbytes, False)
    torch.cuda.synchronize()
    assert bool((small[nbytes // 8 + 4096:] == 0x5A).all())
    big[nbytes:] = 0x5A
    B.adaqp_probe_stream(small[: nbytes // 8 + 4096], big[:nbytes], nbytes, True)
    torch.cuda.synchronize()
    assert bool((big[nbytes:] == 0x5A).all())
    with pytest.raises(B.AdaqpError):
        B.adaqp_probe_stream(big, small, 24, False)                 # not a multiple of 16
    nb = 1_000_000 // 16 * 16
    buf = torch.full((nb + 4096,), 3, dtype=torch.uint8, device=DEV)
    side = torch.zeros(nb // 8 + 4096, dtype=torch.uint8, device=DEV)
    buf[nb:] = 0x5A
    B.adaqp_probe_stream(side, buf[:nb], nb, 2)                     # in place; xor with zeros changes nothing
    torch.cuda.synchronize()
    assert bool((buf[nb:] == 0x5A).all()) and bool((buf[:nb] == 3).all())
    with pytest.raises(B.AdaqpError):
        B.adaqp_probe_stream(side, buf[:nb], nb, 3)


@pytest.mark.parametrize("dim", [128, 256, 512])
def test_backward_receive_twin_touches_only_the_destination_rows(dim):
    _say(f"probe backward receive twin dim={dim}")
    rng = np.random.default_rng(dim)
    n_rows, n = 300, 700
    bits = rng.choice(np.array([2, 4, 8], dtype=np.uint8), size=n)
    peer = np.sort(rng.integers(0, 5, size=n)).astype(np.int32)
    perm, off, pbp = B.adaqp_plan_layout(dim, bits, peer, 5)
    s_bits = np.ascontiguousarray(bits[perm])
    packed = rng.integers(1, 256, size=int(pbp[-1]), dtype=np.uint8)
    params = rng.standard_normal((n, 2), dtype=np.float32)
    dst = rng.integers(100, 250, size=n).astype(np.int32)
    order, seg_ptr = B.adaqp_plan_recv_segments(dst)
    grad0 = rng.standard_normal((n_rows, dim), dtype=np.float32)
    got = torch.from_numpy(grad0).to(DEV)
    B.adaqp_probe_unpack_dequant_add(torch.from_numpy(packed).to(DEV), torch.from_numpy(params).to(DEV),
                                     torch.from_numpy(s_bits).to(DEV), torch.from_numpy(off).to(DEV),
                                     torch.from_numpy(dst).to(DEV), torch.from_numpy(order).to(DEV),
                                     torch.from_numpy(seg_ptr).to(DEV), dim, got)
    torch.cuda.synchronize()
    g = got.cpu().numpy().view(np.uint32)
    touched = np.zeros(n_rows, dtype=bool)
    touched[dst] = True
    assert np.array_equal(g[~touched], grad0.view(np.uint32)[~touched]), "a row no message names was written"
    assert not np.array_equal(g[touched], grad0.view(np.uint32)[touched])
    with pytest.raises(B.AdaqpError):                               # 600 columns: not the twin's shape
        wide = torch.zeros((n_rows, 608), dtype=torch.float32, device=DEV)
        B.adaqp_probe_unpack_dequant_add(torch.from_numpy(packed).to(DEV), torch.from_numpy(params).to(DEV),
                                         torch.from_numpy(s_bits).to(DEV), torch.from_numpy(off).to(DEV),
                                         torch.from_numpy(dst).to(DEV), torch.from_numpy(order).to(DEV),
                                         torch.from_numpy(seg_ptr).to(DEV), 600, wide[:, :600])
