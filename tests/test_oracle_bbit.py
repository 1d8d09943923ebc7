"""Pins for the oracle's b-bit quantizer / dequantizer (Sec. 3.2, Eq. 3-5 with
B = 2^b - 1; bit-width study of Sec. 4.3; Theorem 1) and its half-precision wire.

The pins are: words packed by hand from the format statement, facts that hold for
every seed (extreme elements, values on the grid, one-bin error bound), closed-form
moments of stochastic rounding, agreement with the 1-bit quantizer at b = 1 away
from ties, and numpy's own binary16 conversion for the half-precision wire.
"""
import numpy as np
import pytest

BITS = (1, 2, 4, 8)


def codes_of(packed, d, bits):
    """Independent unpack from the format statement: code of column c = bits
    [b (c mod 64/b), +b) of word c // (64/b)."""
    per = 64 // bits
    c = np.arange(d)
    words = packed[:, c // per]
    return ((words >> np.uint64(bits) * (c % per).astype(np.uint64)) & np.uint64((1 << bits) - 1)).astype(np.int64)


def test_pack_hand_examples(oracle):
    # values that sit on the grid (min 0, max B) are their own codes for every seed
    # b = 2, d = 5: codes 0,3,1,2,3 -> 0 | 3<<2 | 1<<4 | 2<<6 | 3<<8 = 0x39c
    x = np.array([[0, 3, 1, 2, 3]], np.float32)
    p, s, z = oracle.quantize_bbit(x, 5, 1, 2, seed=11, stream=0)
    assert p.shape == (1, 1) and int(p[0, 0]) == 0x39C
    assert s.tolist() == [1.0] and z.tolist() == [0.0]
    # b = 4, d = 17: codes 0..15 fill word 0 nibble by nibble, the 17th opens word 1
    x = np.array([list(range(16)) + [15]], np.float32)
    p, s, z = oracle.quantize_bbit(x, 17, 1, 4, seed=3, stream=2)
    assert p.shape == (1, 2)
    assert int(p[0, 0]) == 0xFEDCBA9876543210 and int(p[0, 1]) == 0xF
    # b = 8, d = 9: bytes in column order, least significant first
    x = np.array([[0, 255, 1, 2, 3, 4, 5, 6, 128]], np.float32)
    p, s, z = oracle.quantize_bbit(x, 9, 1, 8, seed=4, stream=1)
    assert p.shape == (1, 2)
    assert int(p[0, 0]) == 0x060504030201FF00 and int(p[0, 1]) == 0x80
    # b = 1 reduces to one bit per column
    x = np.array([[0, 1, 1]], np.float32)
    p, s, z = oracle.quantize_bbit(x, 3, 1, 1, seed=5, stream=0)
    assert int(p[0, 0]) == 0x6


@pytest.mark.parametrize("bits", BITS)
@pytest.mark.parametrize("d", [1, 2, 7, 8, 9, 31, 32, 33, 63, 64, 65, 100, 256, 602])
def test_grid_values_are_fixed_points(oracle, bits, d):
    """x = mn + j * step with exactly representable step: frac(hbar) = 0, so the code
    is j whatever the random draw; dequantisation returns x bit for bit."""
    B = (1 << bits) - 1
    rng = np.random.default_rng(100 * bits + d)
    j = rng.integers(0, B + 1, size=(6, d))
    if d >= 2:
        j[:, 0] = 0
        j[:, -1] = B
    for mn, step in ((0.0, 1.0), (-4.0, 0.5), (3.0, 0.25)):
        x = (mn + step * j).astype(np.float32)
        for seed in (1, 2, 3):
            p, s, z = oracle.quantize_bbit(x, d, 6, bits, seed=seed, stream=seed)
            assert p.shape[1] == (d * bits + 63) // 64
            got = codes_of(p, d, bits)
            if d >= 2:
                assert np.array_equal(got, j)
                assert np.all(s == np.float32(step)) and np.all(z == np.float32(mn))
            else:
                assert not got.any() and not s.any()
            # padding codes are zero
            per = 64 // bits
            full = codes_of(p, p.shape[1] * per, bits)
            assert not full[:, d:].any()
            out = np.full((8, d), np.nan, np.float32)
            oracle.dequantize_bbit_fwd(p, s, z, d, bits, out, 1)
            assert np.array_equal(out[1:7], x)
            assert np.isnan(out[0]).all() and np.isnan(out[7]).all()


@pytest.mark.parametrize("bits", BITS)
def test_extremes_and_one_bin_bound(oracle, bits):
    """For every seed: the arg-min element gets code 0, the arg-max element code B, every
    code is within [0, B], and no element moves by more than one bin (Eq. 4 rounds to a
    neighbouring integer)."""
    B = (1 << bits) - 1
    rng = np.random.default_rng(bits)
    d = 200
    x = (rng.standard_normal((50, d)) * np.exp(rng.standard_normal((50, 1)) * 2)).astype(np.float32)
    for seed in range(5):
        p, s, z = oracle.quantize_bbit(x, d, 50, bits, seed=seed, stream=9)
        q = codes_of(p, d, bits)
        assert q.min() >= 0 and q.max() <= B
        r = np.arange(50)
        assert np.all(q[r, x.argmin(1)] == 0)
        assert np.all(q[r, x.argmax(1)] == B)
        assert np.array_equal(z, x.min(1))
        rng64 = x.max(1).astype(np.float64) - x.min(1)
        assert np.allclose(s.astype(np.float64) * B, rng64, rtol=3e-7, atol=0)
        # "scale is the ratio of the range to B": one single-precision division
        assert np.array_equal(s, (x.max(1) - x.min(1)) / np.float32(B))
        out = np.empty((50, d), np.float32)
        oracle.dequantize_bbit_fwd(p, s, z, d, bits, out, 0)
        bin_w = s.astype(np.float64)[:, None]
        assert np.all(np.abs(out.astype(np.float64) - x) <= bin_w * (1 + 1e-5) + 1e-6 * np.abs(x))
        # recovered values stay inside the row's range up to rounding of the top level
        top = np.maximum(np.abs(x.min(1)), np.abs(x.max(1)))[:, None]
        assert np.all(out >= x.min(1)[:, None])
        assert np.all(out <= x.max(1)[:, None] + 4 * np.spacing(top.astype(np.float32)))


@pytest.mark.parametrize("bits", BITS)
def test_unbiased_with_closed_form_variance(oracle, bits):
    """Theorem 1: E[recovered] = h; for stochastic rounding between two neighbouring
    levels the variance is step^2 f (1 - f), f = frac(hbar)."""
    B = (1 << bits) - 1
    d, S = 64, 3000
    rng = np.random.default_rng(40 + bits)
    row = rng.uniform(-1, 2, size=d).astype(np.float32)
    x = np.repeat(row[None], S, axis=0)              # S wire rows = S independent draws
    p, s, z = oracle.quantize_bbit(x, d, S, bits, seed=77, stream=5)
    out = np.empty((S, d), np.float32)
    oracle.dequantize_bbit_fwd(p, s, z, d, bits, out, 0)
    step = (row.max().astype(np.float64) - row.min()) / B
    hbar = (row.astype(np.float64) - row.min()) / step
    f = hbar - np.floor(hbar)
    var = step ** 2 * f * (1 - f)
    mean = out.astype(np.float64).mean(0)
    assert np.all(np.abs(mean - row) <= 5 * np.sqrt(var / S) + 1e-6)
    emp = out.astype(np.float64).var(0)
    assert np.all(np.abs(emp - var) <= 0.15 * step ** 2 * 0.25 + 1e-9)
    assert emp.max() <= step ** 2 / 4 * 1.1
    # the codes are the two neighbours of hbar and nothing else
    q = codes_of(p, d, bits)
    assert np.all((q >= np.floor(hbar - 1e-4)) & (q <= np.ceil(hbar + 1e-4)))


def test_one_bit_agrees_with_the_one_bit_quantizer(oracle):
    """At b = 1 both quantizers realise [u < hbar]; they may differ only where u and hbar
    coincide to within the rounding of the two formulations."""
    rng = np.random.default_rng(8)
    n, d = 400, 96
    x = (rng.standard_normal((n, d)) * 3).astype(np.float32)
    p1, s1, z1 = oracle.quantize_1bit(x, d, n, seed=21, stream=4)
    pb, sb, zb = oracle.quantize_bbit(x, d, n, 1, seed=21, stream=4)
    assert np.array_equal(s1, sb) and np.array_equal(z1, zb)
    diff = codes_of(p1, d, 1) != codes_of(pb, d, 1)
    hbar = (x.astype(np.float64) - z1[:, None]) / s1[:, None]
    u = np.array([[oracle.uniform24(21, 4, i, c) for c in range(d)] for i in range(n)]) / 2.0 ** 24
    assert np.all(np.abs(u - hbar)[diff] < 2.0 ** -21)
    assert diff.mean() < 1e-3
    out1 = np.empty((n, d), np.float32); outb = np.empty((n, d), np.float32)
    oracle.dequantize_1bit_fwd(p1, s1, z1, d, out1, 0)
    oracle.dequantize_bbit_fwd(p1, s1, z1, d, 1, outb, 0)
    assert np.array_equal(out1, outb)


@pytest.mark.parametrize("bits", BITS)
def test_degenerate_rows(oracle, bits):
    B = (1 << bits) - 1
    d = 64
    x = np.zeros((6, d), np.float32)
    x[0] = 2.5                       # constant
    x[1] = -0.0                      # negative zeros
    x[2, 5] = 2.0 ** -140            # range far below the normal numbers
    x[3, ::2] = 2.0 ** 125; x[3, 1::2] = -(2.0 ** 125)   # range near the top
    x[4] = 1e-30; x[4, 1] = 3e-30                         # small normal range, one interior value
    x[4, 2] = 2e-30
    x[5] = np.float32(1.0); x[5, 3] = np.nextafter(np.float32(1.0), np.float32(2.0))
    for seed in range(4):
        p, s, z = oracle.quantize_bbit(x, d, 6, bits, seed=seed, stream=1)
        q = codes_of(p, d, bits)
        assert q.min() >= 0 and q.max() <= B
        assert p.shape[1] * 64 == d * bits                 # no padding: every bit is a code bit
        out = np.empty((6, d), np.float32)
        oracle.dequantize_bbit_fwd(p, s, z, d, bits, out, 0)
        assert not q[0].any() and not q[1].any()
        assert np.array_equal(out[0], x[0])
        assert np.array_equal(out[1].view(np.uint32), np.zeros(d, np.uint32))     # -0 -> +0
        for r in (2, 3, 5):          # two-valued rows: low value -> 0, high value -> B
            hi = x[r] == x[r].max()
            assert np.all(q[r][hi] == B) and not q[r][~hi].any()
        assert np.all(np.isfinite(out))
        assert q[4, 0] == 0 and q[4, 1] == B
        assert abs(int(q[4, 2]) - B / 2) <= 0.51           # midpoint: one of its two neighbours


def test_backward_integrate_order(oracle):
    """Duplicates of one destination are added one after the other in wire-row order, in
    single precision (Alg. 2, integrate)."""
    rng = np.random.default_rng(3)
    d, n, bits = 24, 40, 4
    x = (rng.standard_normal((n, d)) * 1e3).astype(np.float32)
    p, s, z = oracle.quantize_bbit(x, d, n, bits, seed=1, stream=1)
    deq = np.empty((n, d), np.float32)
    oracle.dequantize_bbit_fwd(p, s, z, d, bits, deq, 0)
    dst = rng.integers(0, 5, size=n).astype(np.int32)
    J0 = rng.standard_normal((5, d)).astype(np.float32)
    J = J0.copy()
    oracle.dequantize_bbit_bwd(p, s, z, d, bits, J, dst)
    ref = J0.copy()
    for i in range(n):
        ref[dst[i]] = ref[dst[i]] + deq[i]               # numpy float32 adds, same order
    assert np.array_equal(J, ref)
    rev = J0.copy()
    for i in reversed(range(n)):
        rev[dst[i]] = rev[dst[i]] + deq[i]
    assert not np.array_equal(J, rev)                    # the order is observable


def test_gather_offset_and_window(oracle):
    """idx / row_offset select source rows; wire_row0 shifts the random stream so that a
    window of an exchange reproduces the same codes."""
    rng = np.random.default_rng(5)
    src = rng.standard_normal((30, 20)).astype(np.float32)
    idx = rng.integers(0, 30, size=12).astype(np.int32)
    pa, sa, za = oracle.quantize_bbit(src, 20, 12, 4, seed=9, stream=2, idx=idx)
    pb, sb, zb = oracle.quantize_bbit(np.ascontiguousarray(src[idx]), 20, 12, 4, seed=9, stream=2)
    assert np.array_equal(pa, pb) and np.array_equal(sa, sb) and np.array_equal(za, zb)
    pc, sc, zc = oracle.quantize_bbit(src, 20, 5, 4, seed=9, stream=2, row_offset=7, wire_row0=3)
    pd, sd, zd = oracle.quantize_bbit(np.ascontiguousarray(src[4:12]), 20, 8, 4, seed=9, stream=2)
    assert np.array_equal(pc, pd[3:]) and np.array_equal(sc, sd[3:])
    # a wider leading dimension than d
    pe, se, ze = oracle.quantize_bbit(src, 13, 12, 4, seed=9, stream=2, idx=idx)
    pf, sf, zf = oracle.quantize_bbit(np.ascontiguousarray(src[idx][:, :13]), 13, 12, 4, seed=9, stream=2)
    assert np.array_equal(pe, pf)


# ---- half-precision wire ------------------------------------------------------------

def test_fp16_matches_numpy_conversion(oracle):
    rng = np.random.default_rng(16)
    special = np.array([0.0, -0.0, 1.0, -1.0, 65504.0, 65519.99, 65520.0, 70000.0, -1e9, np.inf, -np.inf,
                        2.0 ** -14, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001, 2.0 ** -26, 1.5 * 2.0 ** -24,
                        2.5 * 2.0 ** -24, 1.0 + 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -11,
                        2047.5, 2048.5, 0.1, 1e-7, 3.3e-5, 6.1e-5], np.float32)
    rnd = (rng.standard_normal(200000) * np.exp(rng.standard_normal(200000) * 6)).astype(np.float32)
    bits = rng.integers(0, 2 ** 32, size=200000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    bits = bits[np.isfinite(bits)]
    x = np.concatenate([special, rnd, bits])
    d = 7
    n = x.size // d
    x = np.ascontiguousarray(x[: n * d].reshape(n, d))
    w = oracle.convert_fp16(x, d, n)
    assert w.shape == (n, 8) and not w[:, d:].any()
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(w[:, :d], ref)
    out = np.full((n + 1, d), np.nan, np.float32)
    oracle.recover_fp16_fwd(w, d, out, 1)
    assert np.array_equal(out[1:].view(np.uint32), ref.view(np.float16).astype(np.float32).view(np.uint32))


def test_fp16_every_half_decodes(oracle):
    h = np.arange(65536, dtype=np.uint16)
    w = np.ascontiguousarray(h.reshape(-1, 4))
    out = np.empty((w.shape[0], 4), np.float32)
    oracle.recover_fp16_fwd(w, 4, out, 0)
    ref = h.view(np.float16).astype(np.float32).reshape(-1, 4)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(out), nan)
    assert np.array_equal(out[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    # and encodes back to itself
    fin = np.ascontiguousarray(np.where(nan, 0.0, ref).astype(np.float32))
    w2 = oracle.convert_fp16(fin, 4, fin.shape[0])
    assert np.array_equal(w2[~nan], w[~nan])


def test_fp16_backward_integrate(oracle):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((20, 10)).astype(np.float32)
    w = oracle.convert_fp16(x, 10, 20)
    dst = rng.integers(0, 4, size=20).astype(np.int32)
    J0 = rng.standard_normal((4, 10)).astype(np.float32)
    J = J0.copy()
    oracle.recover_fp16_bwd(w, 10, J, dst)
    ref = J0.copy()
    half = x.astype(np.float16).astype(np.float32)
    for i in range(20):
        ref[dst[i]] = ref[dst[i]] + half[i]
    assert np.array_equal(J, ref)
