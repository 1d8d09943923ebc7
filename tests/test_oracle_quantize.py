"""Pins for the oracle's quantizer / dequantizer (Sec. 3.2, Eq. 3-5; Theorem 1).

None of these re-type the oracle's formula: they use hand-packed words, brute-force
extrema, facts that hold for every seed, closed-form moments of the rounding, the
paper's own volume table, and the literal real-number form of Eq. 3-4 in float64.
"""
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def unpack_bits(packed, d):
    """Independent unpack: numpy's unpackbits on the little-endian bytes."""
    b = np.unpackbits(packed.view(np.uint8).reshape(packed.shape[0], -1), axis=1,
                      bitorder="little")
    return b[:, :d], b[:, d:]


def binary_rows(rng, n, d):
    """0/1 rows that contain both values: these quantise to themselves for every seed
    (the min element always rounds down, the max element always rounds up)."""
    b = rng.integers(0, 2, size=(n, d)).astype(np.float32)
    if d >= 2:
        b[:, 0] = 0.0
        b[:, d - 1] = 1.0
    return b


def test_pack_hand_examples(oracle):
    # d = 3: row (0, 1, 1) -> bits 0b110 = 0x6 ; row (0, 0, 1) -> 0b100 = 0x4
    x = np.array([[0, 1, 1], [0, 0, 1]], np.float32)
    p, s, z = oracle.quantize_1bit(x, 3, 2, seed=5, stream=0)
    assert p.shape == (2, 1) and p.dtype == np.uint64
    assert [int(v) for v in p[:, 0]] == [0x6, 0x4]
    assert s.tolist() == [1.0, 1.0] and z.tolist() == [0.0, 0.0]
    # d = 65: ones at columns 1, 63, 64 -> word0 = 2^63 + 2, word1 = 1
    x = np.zeros((2, 65), np.float32)
    x[0, [1, 63, 64]] = 1.0
    x[1, [0, 2, 62]] = 1.0
    p, s, z = oracle.quantize_1bit(x, 65, 2, seed=9, stream=3)
    assert p.shape == (2, 2)
    assert int(p[0, 0]) == 0x8000000000000002 and int(p[0, 1]) == 0x1
    assert int(p[1, 0]) == 0x4000000000000005 and int(p[1, 1]) == 0x0


@pytest.mark.parametrize("d", list(range(2, 131)) + [255, 256, 257, 602])
def test_pack_unpack_identity_and_padding(oracle, d):
    rng = np.random.default_rng(d)
    b = binary_rows(rng, 7, d)
    p, s, z = oracle.quantize_1bit(b, d, 7, seed=d, stream=1)
    assert p.shape[1] == (d + 63) // 64
    bits, pad = unpack_bits(p, d)
    assert np.array_equal(bits, b.astype(np.uint8))
    assert not pad.any()
    out = np.full((9, d), np.nan, np.float32)
    oracle.dequantize_1bit_fwd(p, s, z, d, out, 1)
    assert np.array_equal(out[1:8], b)            # unpack(pack(b)) == b, placed at the offset
    assert np.isnan(out[0]).all() and np.isnan(out[8]).all()


def test_extrema_and_metadata_bruteforce(oracle):
    rng = np.random.default_rng(1)
    for d in (1, 2, 5, 64, 100, 602):
        x = (rng.standard_normal((50, d)) * np.exp(rng.standard_normal((50, 1)) * 2)).astype(
            np.float32)
        p, s, z = oracle.quantize_1bit(x, d, 50, seed=1, stream=0)
        assert np.array_equal(z, x.min(1))
        assert np.array_equal(s, x.max(1) - x.min(1))          # one float subtraction
        assert (s >= 0).all()


def test_gather_index_and_offset(oracle):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((40, 70)).astype(np.float32)
    idx = rng.integers(0, 40, 25).astype(np.int32)              # duplicates on purpose
    a = oracle.quantize_1bit(x, 70, 25, 77, 4, idx=idx)
    b = oracle.quantize_1bit(np.ascontiguousarray(x[idx]), 70, 25, 77, 4)
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    c = oracle.quantize_1bit(x, 70, 10, 77, 4, row_offset=30)
    e = oracle.quantize_1bit(np.ascontiguousarray(x[30:]), 70, 10, 77, 4)
    for u, v in zip(c, e):
        assert np.array_equal(u, v)
    # a window of an exchange recomputed on its own gives the same rows
    h = oracle.quantize_1bit(np.ascontiguousarray(x[idx[7:19]]), 70, 12, 77, 4, wire_row0=7)
    for u, v in zip(a, h):
        assert np.array_equal(u[7:19], v)
    # leading dimension larger than d: only the first d columns are read
    f = oracle.quantize_1bit(x, 33, 40, 77, 4)
    g = oracle.quantize_1bit(np.ascontiguousarray(x[:, :33]), 33, 40, 77, 4)
    for u, v in zip(f, g):
        assert np.array_equal(u, v)


def test_constant_row_exact(oracle):
    for val in (0.0, -0.0, 3.25, -1e-30, 7e20):
        x = np.full((3, 77), val, np.float32)
        p, s, z = oracle.quantize_1bit(x, 77, 3, seed=4, stream=2)
        assert not p.any() and (s == 0).all()
        out = np.empty((3, 77), np.float32)
        oracle.dequantize_1bit_fwd(p, s, z, 77, out, 0)
        assert np.array_equal(out, x)
        # -0 is canonicalised: the stored zero-point is +0
        assert not np.signbit(z).any() or val != 0.0


def test_argmin_zero_argmax_one_every_seed(oracle):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((64, 90)).astype(np.float32)
    amin, amax = x.argmin(1), x.argmax(1)
    for seed in range(200):
        p, s, z = oracle.quantize_1bit(x, 90, 64, seed=seed * 7919, stream=seed % 5)
        bits, _ = unpack_bits(p, 90)
        assert not bits[np.arange(64), amin].any()
        assert bits[np.arange(64), amax].all()


def test_two_element_rows_round_trip_every_seed(oracle):
    rng = np.random.default_rng(4)
    x = rng.standard_normal((100, 2)).astype(np.float32) * 10
    for seed in range(50):
        p, s, z = oracle.quantize_1bit(x, 2, 100, seed=seed, stream=0)
        out = np.empty_like(x)
        oracle.dequantize_1bit_fwd(p, s, z, 2, out, 0)
        mn, mx = x.min(1), x.max(1)
        lo, hi = out.min(1), out.max(1)
        assert np.array_equal(lo, mn)
        assert np.array_equal(hi, (mn + (mx - mn)).astype(np.float32))
        assert np.array_equal(out.argmax(1), x.argmax(1))


def test_dequant_values_and_range(oracle):
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((200, 130)) * np.exp(3 * rng.standard_normal((200, 1)))).astype(
        np.float32)
    x[0, :] = 1.5
    x[0, 0] = -(2.0 ** 24)          # max is not recovered exactly: 1 ulp slack case
    p, s, z = oracle.quantize_1bit(x, 130, 200, seed=11, stream=0)
    out = np.empty_like(x)
    oracle.dequantize_1bit_fwd(p, s, z, 130, out, 0)
    lo = x.min(1, keepdims=True)
    hi = x.max(1, keepdims=True)
    top = (z + s).astype(np.float32)[:, None]
    assert ((out == z[:, None]) | (out == top)).all()           # two levels only
    slack = np.spacing(np.maximum(np.abs(lo), np.abs(hi)).astype(np.float32))
    assert (out >= lo).all() and (out <= hi + slack).all()


def test_backward_accumulate_order_and_duplicates(oracle):
    rng = np.random.default_rng(6)
    d, n = 70, 60
    g = rng.standard_normal((n, d)).astype(np.float32)
    p, s, z = oracle.quantize_1bit(g, d, n, seed=3, stream=5)
    deq = np.empty_like(g)
    oracle.dequantize_1bit_fwd(p, s, z, d, deq, 0)
    dst = rng.integers(0, 9, n).astype(np.int32)
    J0 = rng.standard_normal((12, d)).astype(np.float32)
    J = J0.copy()
    oracle.dequantize_1bit_bwd(p, s, z, d, J, dst)
    ref = J0.copy()
    for i in range(n):                                          # sequential float32 adds
        ref[dst[i]] = (ref[dst[i]] + deq[i]).astype(np.float32)
    assert np.array_equal(J, ref)
    assert np.array_equal(J[9:], J0[9:])                        # untouched rows
    # against exact arithmetic: the float32 chain stays within n ulps of the true sum
    exact = J0.astype(np.float64)
    np.add.at(exact, dst, deq.astype(np.float64))
    assert np.abs(J - exact).max() <= 64 * np.spacing(np.float32(np.abs(exact).max()))


def test_unbiased_and_variance_closed_form(oracle):
    """Theorem 1: E[dequant(quant(h))] = h; per element Var = range^2 p (1-p)."""
    d, S = 64, 4000
    rng = np.random.default_rng(7)
    x = rng.uniform(-1.0, 3.0, size=(1, d)).astype(np.float32)
    x[0, 0], x[0, 1] = -1.0, 3.0
    xs = np.repeat(x, S, axis=0)                                # one wire row index per trial
    acc = np.zeros(d)
    acc2 = np.zeros(d)
    trials = 0
    for seed in range(8):
        p, s, z = oracle.quantize_1bit(xs, d, S, seed=1000 + seed, stream=seed)
        out = np.empty_like(xs)
        oracle.dequantize_1bit_fwd(p, s, z, d, out, 0)
        acc += out.astype(np.float64).sum(0)
        acc2 += (out.astype(np.float64) ** 2).sum(0)
        trials += S
    mean = acc / trials
    var = acc2 / trials - mean ** 2
    rngw = 4.0
    pr = (x[0].astype(np.float64) + 1.0) / rngw
    sigma = rngw * np.sqrt(pr * (1 - pr) / trials)
    assert (np.abs(mean - x[0]) <= 5 * sigma + 1e-6).all()
    true_var = rngw ** 2 * pr * (1 - pr)
    # variance of a sample variance of a two-point law: generous 6-sigma band
    assert (np.abs(var - true_var) <= 6 * rngw ** 2 * np.sqrt(1.0 / trials) + 1e-9).all()


def test_theorem1_row_variance(oracle):
    """Theorem 1's Var = D * range^2 / (6 B^2) under uniform fractions, B = 1."""
    D, S = 512, 3000
    rng = np.random.default_rng(8)
    x = rng.uniform(0.0, 1.0, size=(1, D)).astype(np.float32)
    x[0, 0], x[0, 1] = 0.0, 1.0
    xs = np.repeat(x, S, axis=0)
    p, s, z = oracle.quantize_1bit(xs, D, S, seed=99, stream=1)
    out = np.empty_like(xs)
    oracle.dequantize_1bit_fwd(p, s, z, D, out, 0)
    err2 = ((out.astype(np.float64) - x) ** 2).sum(1)           # ||htilde - h||^2 per trial
    got = err2.mean()
    want = D * 1.0 / 6.0
    # the realised fractions are one sample of U(0,1)^D: sum p(1-p) has sd ~ sqrt(D/180)
    assert abs(got - want) <= 5 * np.sqrt(D / 180.0) + 5 * err2.std() / np.sqrt(S)


def test_literal_eq3_eq4_in_float64(oracle):
    """The paper's form, hbar = (h - min)/(max - min), bit = [u < hbar], evaluated in
    float64, must give the same bits except where u and hbar tie to ~2^-22."""
    rng = np.random.default_rng(9)
    n, d = 400, 96
    x = (rng.standard_normal((n, d)) * np.exp(rng.standard_normal((n, 1)))).astype(np.float32)
    p, s, z = oracle.quantize_1bit(x, d, n, seed=321, stream=6)
    bits, _ = unpack_bits(p, d)
    u = np.array([[oracle.uniform24(321, 6, i, c) for c in range(d)] for i in range(n)],
                 np.float64) / 2.0 ** 24
    mn = x.min(1, keepdims=True).astype(np.float64)
    mx = x.max(1, keepdims=True).astype(np.float64)
    hbar = (x.astype(np.float64) - mn) / (mx - mn)
    lit = (u < hbar).astype(np.uint8)
    diff = bits != lit
    assert (np.abs(u - hbar)[diff] < 2.0 ** -22).all()
    assert diff.mean() < 1e-5


def test_monotone_in_value(oracle):
    """With the random draws fixed, raising an element can only turn its bit on."""
    rng = np.random.default_rng(10)
    d = 80
    base = rng.uniform(0, 1, size=(300, d)).astype(np.float32)
    base[:, 0], base[:, 1] = 0.0, 1.0                           # pins min / max
    up = base.copy()
    up[:, 2:] = np.minimum(1.0, up[:, 2:] + rng.uniform(0, 0.3, size=(300, d - 2))).astype(
        np.float32)
    pa, _, _ = oracle.quantize_1bit(base, d, 300, seed=5, stream=5)
    pb, _, _ = oracle.quantize_1bit(up, d, 300, seed=5, stream=5)
    assert not (pa & ~pb).any()


def test_uniform24_statistics(oracle):
    """The draws behind the rounding: range, chi-square uniformity, and no coupling
    between neighbouring columns, rows, streams or seeds."""
    n = 1 << 16
    cols = np.array([oracle.uniform24(42, 3, 17, c) for c in range(n)], np.int64)
    rows = np.array([oracle.uniform24(42, 3, r, 5) for r in range(n)], np.int64)
    strm = np.array([oracle.uniform24(42, s_, 17, 5) for s_ in range(n)], np.int64)
    seed = np.array([oracle.uniform24(sd * 2**32 + 1, 3, 17, 5) for sd in range(n)], np.int64)
    for name, k in (("cols", cols), ("rows", rows), ("streams", strm), ("seeds", seed)):
        assert k.min() >= 0 and k.max() < 2 ** 24, name
        hist = np.bincount(k >> 16, minlength=256)              # 256 buckets, 255 dof
        chi2 = ((hist - n / 256) ** 2 / (n / 256)).sum()
        assert chi2 < 255 + 6 * np.sqrt(2 * 255), (name, chi2)
        u = k / 2.0 ** 24
        assert abs(u.mean() - 0.5) < 5 / np.sqrt(12 * n), name
        lag = np.corrcoef(u[:-1], u[1:])[0, 1]
        assert abs(lag) < 5 / np.sqrt(n), (name, lag)
        for bit in range(24):
            frac = ((k >> bit) & 1).mean()
            assert abs(frac - 0.5) < 5 * 0.5 / np.sqrt(n), (name, bit, frac)
    assert abs(np.corrcoef(cols / 2.0 ** 24, rows / 2.0 ** 24)[0, 1]) < 5 / np.sqrt(n)
    # different keys give different streams
    assert (cols != np.array([oracle.uniform24(42, 4, 17, c) for c in range(64)] * (n // 64))
            ).mean() > 0.99


def test_wire_volume_matches_paper_table(oracle):
    """Main data shrinks 32x when 64 | d (caption: "almost 32x"); side channel is 8 B/row."""
    rows = []
    with open(os.path.join(HERE, "golden", "comm_volume_table.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, fp32, main, ec = line.split()
            rows.append((name, float(fp32), float(main), float(ec)))
    assert len(rows) == 4
    for name, fp32, main, ec in rows:
        assert abs(fp32 / main - 32.0) < 0.06, name             # printed to 0.1 MB
        assert ec < 0.26 * main                                 # "much smaller portions"
    for d in (64, 128, 256, 512):
        assert 4 * d / (8 * oracle.words_per_row(d)) == 32.0
    for d in (100, 602):                                        # padded last word: a bit below 32x
        r = 4 * d / (8 * oracle.words_per_row(d))
        assert 24.0 < r < 32.0
    # side channel relative to main data is 64/d for 64 | d: the table's ratios
    # (0.06 .. 0.25) correspond to exchanged widths between 256 and ~1000 bits
    for name, fp32, main, ec in rows:
        assert 64 / 1100 < ec / main < 64 / 250, name
