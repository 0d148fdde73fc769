"""Pins for the oracle's quantise / pack / unpack / de-quantise (Sec. 2.3 Eq. 4-5, Theorem 1, App. A.1).

Each test checks the oracle against something other than itself: hand-derived closed forms, invariants the
paper states, numpy's own bit packing, float64 re-derivations from the published (Z, S).
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
WIDTHS = (2, 4, 8)


def _single_width(oracle, rows, b, seed=0, want_codes=True):
    """Quantise every row of `rows` (2-D fp32) at width b; one peer, identity send list."""
    rows = np.ascontiguousarray(rows, dtype=np.float32)
    n, dim = rows.shape
    bits = np.full(n, b, dtype=np.uint8)
    perm, off, pbp = oracle.plan_layout(dim, bits, np.zeros(n, dtype=np.int32), 1)
    assert np.array_equal(perm, np.arange(n))
    packed, params, codes = oracle.quantize_pack(rows, dim, np.arange(n, dtype=np.int32), bits, off, seed,
                                                 int(pbp[-1]), want_codes=want_codes)
    return packed, params, codes, off


def test_closed_form_rows_and_bytes(oracle):
    pats = {}
    for line in open(os.path.join(GOLDEN, "pack_patterns.txt")):
        if line.strip() and not line.startswith("#"):
            b, hexbytes = line.split()
            pats[int(b)] = bytes.fromhex(hexbytes)
    for b in WIDTHS:
        L = (1 << b) - 1
        row = np.arange(L + 1, dtype=np.float32)[None, :]
        for seed in (0, 1, 7, 2**40 + 3, 2**64 - 1):
            packed, params, codes, _ = _single_width(oracle, row, b, seed)
            assert params[0, 0] == 0.0 and params[0, 1] == 1.0
            assert np.array_equal(codes[0], np.arange(L + 1))
            if b in pats:
                assert packed.tobytes() == pats[b]
            else:
                assert packed.tobytes() == bytes(range(256))
            out = np.full((1, L + 1), np.nan, dtype=np.float32)
            oracle.unpack_dequant(packed, params, np.array([b], np.uint8), np.array([0], np.int64),
                                  np.array([0], np.int32), L + 1, out)
            assert np.array_equal(out, row)


def test_affine_closed_form(oracle):
    # the code grid is invariant under h -> a*h + c for power-of-two a and exactly representable c
    for b in WIDTHS:
        L = (1 << b) - 1
        row = (np.arange(L + 1, dtype=np.float32) * np.float32(0.25) - np.float32(3.0))[None, :]
        packed, params, codes, _ = _single_width(oracle, row, b, seed=5)
        assert params[0, 0] == np.float32(-3.0) and params[0, 1] == np.float32(0.25)
        assert np.array_equal(codes[0], np.arange(L + 1))


def test_code_range_and_endpoints(oracle):
    rng = np.random.default_rng(11)
    for b in WIDTHS:
        L = (1 << b) - 1
        rows = rng.standard_normal((64, 97), dtype=np.float32) * rng.choice([1e-6, 1.0, 3e4], size=(64, 1)).astype(np.float32)
        rows[5] = np.float32(2.5)                              # constant row
        rows[6, :] = 0.0
        rows[6, 3] = -0.0                                      # both zeros
        rows[7] = np.abs(rows[7])                              # non-negative
        rows[8, :50] = 0.0
        for seed in range(20):
            _, params, codes, _ = _single_width(oracle, rows, b, seed)
            assert codes.max() <= L
            amin, amax = rows.argmin(1), rows.argmax(1)
            r = np.arange(rows.shape[0])
            const = rows.max(1) == rows.min(1)
            assert np.all(codes[r, amin] == 0)
            assert np.all(codes[r, amax][~const] == L)
            assert np.all(codes[const] == 0)
            assert np.all(params[const, 1] == 0)
            assert np.array_equal(params[:, 0], rows.min(1) + np.float32(0.0))
            assert not np.signbit(params[6, 0])


def _tiny_range_rows(scale, dim=24, seed=0):
    """Rows whose range is about `scale` around offsets of very different size (0, tiny, ordinary)."""
    rng = np.random.default_rng(seed)
    u = rng.random((6, dim))
    u[:, 0], u[:, 1] = 0.0, 1.0                                # the row's minimum and maximum
    base = np.array([0.0, scale * 8, -scale * 3, 1e-20, 0.0, 0.0])[:, None]
    rows = (base + u * scale).astype(np.float32)
    rows[4] = np.float32(scale)                                # constant row at that size
    rows[5, 1:] = rows[5, 0]                                   # all equal ...
    rows[5, 1] = np.nextafter(rows[5, 0], np.float32(1), dtype=np.float32)     # ... but one element one ulp up
    return rows


@pytest.mark.parametrize("scale", [1e-30, 1e-33, 1e-36, 3e-38, 1e-39, 1e-42, 3e-45])
def test_tiny_and_denormal_ranges(oracle, scale):
    """Eq. 4 at the bottom of fp32: ranges down to denormals.  Either the reciprocal (2^b-1)/range is an fp32
    number and the row is quantised as any other (minimum -> 0, maximum -> 2^b-1, every code within one step of
    the float64 quotient), or it overflows and the row counts as constant (S = 0, codes 0, de-quantised = Z)."""
    flt_max = float(np.finfo(np.float32).max)
    for b in WIDTHS:
        L = (1 << b) - 1
        rows = _tiny_range_rows(scale)
        for seed in (0, 1, 12345):
            packed, params, codes, off = _single_width(oracle, rows, b, seed)
            assert codes.max() <= L
            Z = params[:, 0].astype(np.float64)
            S = params[:, 1].astype(np.float64)
            mn, mx = rows.min(1), rows.max(1)
            rng32 = (mx + np.float32(0)) - (mn + np.float32(0))          # exact in fp32 here (Sterbenz or denormal)
            assert np.array_equal(params[:, 0], mn + np.float32(0))
            for r in range(rows.shape[0]):
                rr = float(rng32[r])
                if rr == 0.0 or L / rr > flt_max:                        # constant, or treated as constant
                    assert S[r] == 0.0 and np.all(codes[r] == 0), (scale, b, r)
                    continue
                assert S[r] == float(np.float32(rng32[r]) / np.float32(L))
                assert codes[r, rows[r].argmin()] == 0 and codes[r, rows[r].argmax()] == L, (scale, b, r)
                x = (rows[r].astype(np.float64) - Z[r]) * (L / rr)       # exact quotient position, float64
                assert np.all(np.abs(codes[r] - x) < 1.0 + 1e-3), (scale, b, r)
            out = np.full_like(rows, np.nan)
            n = rows.shape[0]
            oracle.unpack_dequant(packed, params, np.full(n, b, np.uint8), off, np.arange(n, dtype=np.int32),
                                  rows.shape[1], out)
            assert np.all(np.abs(out.astype(np.float64) - rows) <= np.maximum(S, rng32.astype(np.float64))[:, None]
                          * (1 + 1e-3) + 1e-45)


def test_overshoot_of_top_element_is_clamped(oracle):
    # search for rows where (max - Z) * inv rounds above 2^b - 1 in fp32: the clamp must still give code L
    rng = np.random.default_rng(3)
    found = 0
    for b in WIDTHS:
        L = np.float32((1 << b) - 1)
        lo = rng.standard_normal(20000).astype(np.float32)
        hi = lo + np.abs(rng.standard_normal(20000).astype(np.float32)) + np.float32(1e-3)
        rng32 = (hi + np.float32(0)) - (lo + np.float32(0))
        inv = L / rng32
        over = (hi - lo) * inv > L
        found += int(over.sum())
        idx = np.nonzero(over)[0][:50]
        if idx.size == 0:
            continue
        rows = np.stack([lo[idx], hi[idx], (lo[idx] + hi[idx]) / 2], axis=1).astype(np.float32)
        _, _, codes, _ = _single_width(oracle, rows, int(np.log2(L + 1)), seed=1)
        assert np.all(codes[:, 1] == int(L)) and np.all(codes[:, 0] == 0)
    assert found > 0, "the search should exercise the clamp at least once"


def test_two_point_support_and_error_bound(oracle):
    rng = np.random.default_rng(21)
    rows = rng.standard_normal((40, 301), dtype=np.float32)
    rows[::3] = np.maximum(rows[::3], 0)
    for b in WIDTHS:
        for seed in (0, 99):
            packed, params, codes, off = _single_width(oracle, rows, b, seed)
            Z = params[:, :1].astype(np.float64)
            S = params[:, 1:].astype(np.float64)
            x = (rows.astype(np.float64) - Z) / S                       # Eq. 4 argument in float64
            lo, hi = np.floor(x - 1e-4), np.ceil(x + 1e-4)
            assert np.all(codes >= lo) and np.all(codes <= hi)
            assert np.all(np.abs(codes - x) < 1.0 + 1e-4)
            out = np.zeros_like(rows)
            oracle.unpack_dequant(packed, params, np.full(40, b, np.uint8), off, np.arange(40, dtype=np.int32),
                                  301, out)
            assert np.all(np.abs(out.astype(np.float64) - rows) <= S * (1 + 1e-4))
            # Eq. 5 in float64 from the same codes; two fp32 roundings, each relative to its own operand size
            assert np.all(np.abs(out - (codes * S + Z)) <= 1.3e-7 * (np.abs(codes * S) + np.abs(Z)))


def _moments_over_seeds(oracle, rows, b, n_seeds):
    rows = np.ascontiguousarray(rows, dtype=np.float32)
    n, dim = rows.shape
    bits = np.full(n, b, dtype=np.uint8)
    _, off, pbp = oracle.plan_layout(dim, bits, np.zeros(n, dtype=np.int32), 1)
    idx = np.arange(n, dtype=np.int32)
    s1 = np.zeros((n, dim))
    s2 = np.zeros((n, dim))
    out = np.zeros_like(rows)
    params = None
    for seed in range(n_seeds):
        packed, params, _ = oracle.quantize_pack(rows, dim, idx, bits, off, seed, int(pbp[-1]))
        oracle.unpack_dequant(packed, params, bits, off, idx, dim, out)
        o = out.astype(np.float64)
        s1 += o
        s2 += o * o
    mean = s1 / n_seeds
    var = s2 / n_seeds - mean * mean
    return mean, var, params


@pytest.mark.parametrize("b", WIDTHS)
def test_unbiased_and_variance_bounded_over_1e5_seeds(oracle, b):
    """Theorem 1: E[h^] = h.  Per element the rounding is a Bernoulli(f) step of size S, so the standard
    error of the mean over N seeds is S*sqrt(f(1-f)/N) and Var <= S^2/4.  The 16-bit rounding probability
    (reading R2) adds a bias of at most 2^-16 * S."""
    N = 100_000
    rng = np.random.default_rng(100 + b)
    rows = rng.standard_normal((12, 64), dtype=np.float32)
    rows[1::3] = np.maximum(rows[1::3], 0)
    rows[2::3] *= np.float32(1e-3)
    mean, var, params = _moments_over_seeds(oracle, rows, b, N)
    Z = params[:, :1].astype(np.float64)
    S = params[:, 1:].astype(np.float64)
    x = (rows.astype(np.float64) - Z) / S
    f = x - np.floor(x)
    sigma = S * np.sqrt(f * (1 - f) / N)
    slack = S * 2.0 ** -16 + 4 * np.spacing(np.abs(rows).astype(np.float32)).astype(np.float64)
    err = np.abs(mean - rows)
    # 768 elements: 0.27 % of them (two) lie outside 3 sigma by chance; 1 % leaves room for seven, which a correct
    # implementation exceeds about once in a thousand draws of the rows; none may lie outside 5 sigma
    assert np.all(err <= 5 * sigma + slack)
    assert np.mean(err > 3 * sigma + slack) <= 0.01
    assert np.all(var <= S * S / 4 * 1.02 + 1e-30)
    # the Bernoulli variance itself: S^2 f (1 - f), to a few per cent where it is not tiny
    expect = S * S * f * (1 - f)
    big = f * (1 - f) > 0.05
    assert np.allclose(var[big], expect[big], rtol=0.05)


def test_variance_attains_quarter_bound(oracle):
    # row [0, 0.5, 3] at 2 bits: S = 1, the middle element has fraction 1/2, variance S^2/4
    rows = np.array([[0.0, 0.5, 3.0]], dtype=np.float32)
    mean, var, params = _moments_over_seeds(oracle, rows, 2, 40_000)
    assert params[0, 1] == 1.0
    assert abs(var[0, 1] - 0.25) < 0.005
    assert abs(mean[0, 1] - 0.5) < 0.01
    assert var[0, 0] == 0 and var[0, 2] == 0


@pytest.mark.parametrize("b", WIDTHS)
def test_theorem1_variance_value(oracle, b):
    """Theorem 1: with fractions spread uniformly the variance summed over the row is D * S^2 / 6."""
    D = 4096
    L = (1 << b) - 1
    rng = np.random.default_rng(7 + b)
    row = rng.uniform(0, L, size=D).astype(np.float32)
    row[0], row[1] = 0.0, float(L)                       # pins Z = 0, S = 1
    _, var, params = _moments_over_seeds(oracle, row[None, :], b, 3000)
    S = float(params[0, 1])
    assert S == 1.0
    assert abs(var.sum() / (D * S * S / 6) - 1) < 0.03


def test_pack_matches_numpy_bit_packing_and_round_trips(oracle):
    rng = np.random.default_rng(5)
    dims = list(range(1, 71)) + [128, 300, 602]
    for b in WIDTHS:
        for dim in dims:
            rows = rng.standard_normal((3, dim), dtype=np.float32)
            packed, params, codes, off = _single_width(oracle, rows, b, seed=dim)
            stride = oracle.row_stride(dim, b)
            assert stride == 4 * -(-dim * b // 32)
            assert packed.shape[0] == 3 * stride
            for r in range(3):
                # little-endian bit string built by numpy, independent of the oracle's shifting
                bitmat = ((codes[r][:, None] >> np.arange(b)) & 1).astype(np.uint8).reshape(-1)
                expect = np.packbits(bitmat, bitorder="little")
                got = packed[off[r]: off[r] + stride]
                assert np.array_equal(got[: expect.shape[0]], expect)
                assert np.all(got[expect.shape[0]:] == 0)                       # zero padding
            out = np.zeros_like(rows)
            back = oracle.unpack_dequant(packed, params, np.full(3, b, np.uint8), off,
                                         np.arange(3, dtype=np.int32), dim, out, want_codes=True)
            assert np.array_equal(back, codes)


def test_dequant_scatters_only_listed_rows_and_columns(oracle):
    rng = np.random.default_rng(9)
    dim, ld = 10, 13
    rows = rng.standard_normal((4, dim), dtype=np.float32)
    packed, params, codes, off = _single_width(oracle, rows, 4, seed=2)
    feat = np.full((9, ld), np.float32(-77.0))
    halo = np.array([7, 2, 8, 0], dtype=np.int32)
    oracle.unpack_dequant(packed, params, np.full(4, 4, np.uint8), off, halo, dim, feat)
    untouched = np.ones((9, ld), dtype=bool)
    untouched[halo, :dim] = False
    assert np.all(feat[untouched] == -77.0)
    for t, r in enumerate(halo):
        expect = codes[t].astype(np.float32) * params[t, 1] + params[t, 0]   # numpy fp32: product, then sum
        assert np.array_equal(feat[r, :dim], expect)


def test_gather_uses_send_idx_and_ld(oracle):
    rng = np.random.default_rng(10)
    dim, ld = 9, 12
    feat = rng.standard_normal((20, ld), dtype=np.float32)
    send = np.array([4, 19, 4, 0], dtype=np.int32)               # a node may be sent twice
    bits = np.array([2, 2, 8, 8], dtype=np.uint8)
    off = np.array([0, 4, 8, 20], dtype=np.int64)
    packed, params, codes = oracle.quantize_pack(feat, dim, send, bits, off, 3, 32, want_codes=True)
    for s, r in enumerate(send):
        assert params[s, 0] == feat[r, :dim].min()
        L = (1 << int(bits[s])) - 1
        assert codes[s, feat[r, :dim].argmax()] == L
    # slots 0 and 2 carry the same node but are different messages: independent randomness is allowed,
    # identical parameters up to the width are required
    assert params[0, 0] == params[2, 0]


def test_slot_base_selects_the_same_random_stream(oracle):
    """A run of slots computed on its own (slot_base) gives the bytes it has inside the full computation."""
    rng = np.random.default_rng(12)
    rows = rng.standard_normal((9, 70), dtype=np.float32)
    for b in WIDTHS:
        packed, params, codes, off = _single_width(oracle, rows, b, seed=77)
        stride = oracle.row_stride(70, b)
        for s in (0, 4, 8):
            p1, q1, c1 = oracle.quantize_pack(rows, 70, np.array([s], np.int32), np.array([b], np.uint8),
                                              np.array([0], np.int64), 77, stride, want_codes=True, slot_base=s)
            assert np.array_equal(p1, packed[off[s]: off[s] + stride])
            assert np.array_equal(c1[0], codes[s]) and np.array_equal(q1[0], params[s])
        p0, _, _ = oracle.quantize_pack(rows, 70, np.array([4], np.int32), np.array([b], np.uint8),
                                        np.array([0], np.int64), 77, stride, slot_base=0)
        assert not np.array_equal(p0, packed[off[4]: off[4] + stride])      # slot 0's stream differs from slot 4's


# ------------------------------------------------------------------------------------------------------
# backward receive: de-quantise and add (Sec. 3.1)
# ------------------------------------------------------------------------------------------------------

def test_dequant_add_closed_form_and_order(oracle):
    # a row 0..3 at 2 bits de-quantises to itself; two such messages onto a row of ones give 1 + 2 j
    row = np.arange(4, dtype=np.float32)[None, :]
    packed, params, codes, off = _single_width(oracle, np.repeat(row, 2, 0), 2, seed=3)
    grad = np.ones((3, 6), dtype=np.float32)
    oracle.unpack_dequant_add(packed, params, np.full(2, 2, np.uint8), off, np.array([1, 1], np.int32), 4, grad)
    assert np.array_equal(grad[1, :4], 1 + 2 * np.arange(4)) and np.all(grad[1, 4:] == 1)
    assert np.all(grad[0] == 1) and np.all(grad[2] == 1)


def test_dequant_add_equals_dequant_on_zero_rows_and_is_sequential(oracle):
    rng = np.random.default_rng(31)
    dim = 37
    rows = rng.standard_normal((6, dim), dtype=np.float32)
    for b in WIDTHS:
        packed, params, codes, off = _single_width(oracle, rows, b, seed=b)
        bits = np.full(6, b, np.uint8)
        plain = np.zeros((6, dim), dtype=np.float32)
        oracle.unpack_dequant(packed, params, bits, off, np.arange(6, dtype=np.int32), dim, plain)
        # distinct destinations starting from +0: identical to the plain de-quantisation
        grad = np.zeros((6, dim), dtype=np.float32)
        oracle.unpack_dequant_add(packed, params, bits, off, np.arange(6, dtype=np.int32), dim, grad)
        assert np.array_equal(grad, plain + np.float32(0))
        # all six onto one row: the fp32 sum taken in slot order
        grad = np.full((2, dim), np.float32(0.5))
        oracle.unpack_dequant_add(packed, params, bits, off, np.zeros(6, np.int32), dim, grad)
        want = np.full(dim, np.float32(0.5))
        for t in range(6):
            want = want + plain[t]
        assert np.array_equal(grad[0], want) and np.all(grad[1] == 0.5)
        # a different slot order gives the sum in that order (fp32 addition is not associative)
        perm = np.array([5, 3, 1, 0, 2, 4])
        grad2 = np.full((1, dim), np.float32(0.5))
        oracle.unpack_dequant_add(packed, params[perm], bits, off[perm], np.zeros(6, np.int32), dim, grad2)
        want2 = np.full(dim, np.float32(0.5))
        for t in perm:
            want2 = want2 + plain[t]
        assert np.array_equal(grad2[0], want2)
        assert np.allclose(grad2[0], grad[0], rtol=1e-5, atol=1e-6)


# ------------------------------------------------------------------------------------------------------
# trace for the bit-width assigner: beta_k of Sec. 4.2
# ------------------------------------------------------------------------------------------------------

def test_beta_closed_forms(oracle):
    idx = np.arange(3, dtype=np.int32)
    rows = np.stack([np.arange(16), np.full(16, 2.5), np.arange(16) * 4 - 7]).astype(np.float32)
    w = np.array([1.5, 2.0, 0.25], dtype=np.float32)
    beta = oracle.trace_beta(rows, 16, idx, w)
    assert beta[0] == np.float32(1.5 * 16 * 15 * 15 / 6)          # range 15
    assert beta[1] == 0.0                                          # constant row
    assert beta[2] == np.float32(0.25 * 16 * 60 * 60 / 6)         # range 60
    # (max - min)^2 scaling: a power-of-two factor on the row scales beta by its square, exactly
    assert np.array_equal(oracle.trace_beta(rows * np.float32(4), 16, idx, w), beta * np.float32(16))
    # only the first dim columns count, and the row is found through send_idx
    wide = np.concatenate([rows, np.full((3, 2), 1e6, np.float32)], axis=1)
    assert np.array_equal(oracle.trace_beta(np.ascontiguousarray(wide), 16, idx[::-1].copy(), w[::-1].copy()), beta[::-1])


@pytest.mark.parametrize("b", WIDTHS)
def test_beta_is_the_variance_numerator_of_eq8(oracle, b):
    """Eq. 8 charges message k with beta_k / (2^b - 1)^2.  With alpha^2 summing to 1 that is D S^2 / 6, the
    variance Theorem 1 gives for the de-quantised message; compare with the variance measured over seeds."""
    D, L = 4096, (1 << b) - 1
    rng = np.random.default_rng(70 + b)
    row = rng.uniform(0, L, size=D).astype(np.float32)
    row[0], row[1] = 0.0, float(L)
    beta = oracle.trace_beta(row[None, :], D, np.zeros(1, np.int32), np.ones(1, np.float32))
    _, var, params = _moments_over_seeds(oracle, row[None, :], b, 2000)
    assert abs(var.sum() / (float(beta[0]) / (L * L)) - 1) < 0.04
    S = float(params[0, 1])
    assert abs(float(beta[0]) / (L * L) - D * S * S / 6) <= 1e-6 * D * S * S
