"""GPU parity of the b-bit Low-bit Module (b in {2, 4, 8}) and of the half-precision
wire against the CPU oracle: codes, scale, zero, recovered rows and the backward
accumulate are compared bit for bit."""
import numpy as np
import pytest
import torch

from test_gpu_ops import DEV, bits32, dev, make_rows
from util import join_wire

pytestmark = pytest.mark.gpu


def split_wire_bits(wire, n, d, bits):
    Wb = (d * bits + 63) // 64
    w = np.ascontiguousarray(wire).view(np.uint64)[: n * (Wb + 1)].reshape(n, Wb + 1)
    meta = np.ascontiguousarray(w[:, Wb])
    scale = (meta & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.float32)
    zero = (meta >> np.uint64(32)).astype(np.uint32).view(np.float32)
    return np.ascontiguousarray(w[:, :Wb]), scale, zero


def run_quantize(B, oracle, x, d, n, bits, idx, row_offset, seed, stream, fn):
    W1 = (d * bits + 63) // 64 + 1
    assert B.sylvie_wire_row_words_bits(d, bits) == W1
    wire = torch.full((n * W1 + 3,), -1, dtype=torch.int64, device=DEV)
    fn(dev(x), x.shape[1], d, None if idx is None else dev(idx), row_offset, n, bits, seed, stream, wire)
    torch.cuda.synchronize()
    ref = oracle.quantize_bbit(x, d, n, bits, seed, stream, idx=idx, row_offset=row_offset)
    gw = wire.cpu().numpy()
    pk, sc, zp = split_wire_bits(gw, n, d, bits)
    assert np.array_equal(bits32(sc), bits32(ref[1])), "scale"
    assert np.array_equal(bits32(zp), bits32(ref[2])), "zero"
    bad = np.argwhere(pk != ref[0])
    assert bad.size == 0, ("codes", bad[:4], len(bad))
    assert (gw[n * W1:] == -1).all()
    return wire, ref


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("d", [1, 2, 3, 4, 7, 8, 60, 64, 100, 128, 129, 256, 260, 300, 512, 602, 1024, 1028, 1100])
@pytest.mark.parametrize("kind", ["normal", "edge", "relu", "heavy"])
def test_quantize_bbit_parity(oracle, bits, d, kind):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(d * 31 + len(kind) + bits)
    n_src, n = 300, 517                                        # several tiles + ragged tail
    ld = d + (5 if d % 2 else 0)
    x = make_rows(rng, n_src, ld, kind)
    idx = rng.integers(0, n_src, n).astype(np.int32)
    run_quantize(B, oracle, x, d, n, bits, idx, 0, 0xABCDEF0123456789 + d, 6, B.sylvie_quantize_bbit_fwd)
    run_quantize(B, oracle, x, d, 133, bits, None, 100, 12345 + d, 7, B.sylvie_quantize_bbit_bwd)


def test_quantize_bbit_small_counts_and_one_bit(oracle):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(3)
    x = make_rows(rng, 40, 256, "normal")
    for n in (1, 2, 3, 4, 5, 15, 16, 17):
        run_quantize(B, oracle, x, 256, n, 4, None, 7, 99, 1, B.sylvie_quantize_bbit_fwd)
    # bits = 1 is the 1-bit entry point
    W1 = 5
    a = torch.zeros(30 * W1, dtype=torch.int64, device=DEV)
    b = torch.zeros(30 * W1, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_bbit_fwd(dev(x), 256, 256, None, 3, 30, 1, 5, 2, a)
    B.sylvie_quantize_1bit_fwd(dev(x), 256, 256, None, 3, 30, 5, 2, b)
    assert torch.equal(a, b)
    out_a = torch.zeros(30, 256, device=DEV); out_b = torch.zeros(30, 256, device=DEV)
    B.sylvie_dequantize_bbit_fwd(a, 30, 256, 1, out_a, 256, 0)
    B.sylvie_dequantize_1bit_fwd(b, 30, 256, out_b, 256, 0)
    assert torch.equal(out_a, out_b)
    # n = 0: nothing is written, nothing fails
    p = torch.zeros(8, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_bbit_fwd(dev(x), 256, 256, None, 0, 0, 8, 1, 1, p)
    assert not p.any()


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("d", [1, 3, 4, 64, 100, 128, 256, 260, 602, 1100])
def test_dequantize_bbit_fwd_parity(oracle, bits, d):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(d + bits)
    n = 517
    x = make_rows(rng, n, d, "edge")
    pk, sc, zp = oracle.quantize_bbit(x, d, n, bits, 5, 0)
    for ld, off in ((d, 0), (d + 4, 11), (d + 1, 3)):
        ref = rng.standard_normal((n + 20, ld)).astype(np.float32)
        out = dev(ref)
        oracle.dequantize_bbit_fwd(pk, sc, zp, d, bits, ref, off)
        B.sylvie_dequantize_bbit_fwd(dev(join_wire(pk, sc, zp)), n, d, bits, out, ld, off)
        torch.cuda.synchronize()
        assert np.array_equal(bits32(out.cpu().numpy()), bits32(ref)), (ld, off)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("d", [1, 3, 64, 100, 256, 602])
def test_dequantize_bbit_bwd_parity(oracle, bits, d):
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    rng = np.random.default_rng(d + 1 + bits)
    n, n_dst = 900, 400
    g = make_rows(rng, n, d, "heavy")
    pk, sc, zp = oracle.quantize_bbit(g, d, n, bits, 8, 3)
    dst = rng.integers(0, n_dst - 50, n).astype(np.int32)
    dst[:40] = 17
    ld = d + (3 if d % 2 else 4)
    J = rng.standard_normal((n_dst, ld)).astype(np.float32)
    Jg = dev(J)
    oracle.dequantize_bbit_bwd(pk, sc, zp, d, bits, J, dst)
    sp_, sr, di = GE.scatter_segments(dev(dst))
    B.sylvie_dequantize_bbit_bwd(dev(join_wire(pk, sc, zp)), n, d, bits, Jg, ld, sp_, sr,
                                 int(di.numel()), di)
    torch.cuda.synchronize()
    assert np.array_equal(bits32(Jg.cpu().numpy()), bits32(J))


@pytest.mark.parametrize("d", [1, 3, 4, 7, 64, 100, 256, 602, 1100])
def test_fp16_wire_parity(oracle, d):
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    rng = np.random.default_rng(d)
    n_src, n = 300, 517
    ld = d + (5 if d % 2 else 0)
    x = make_rows(rng, n_src, ld, "heavy")
    x[0, : min(d, 6)] = np.array([65504.0, 65520.0, 1e-8, 6e-8, -2.0 ** -24, 1.0 + 2.0 ** -11], np.float32)[: min(d, 6)]
    idx = rng.integers(0, n_src, n).astype(np.int32)
    idx[0] = 0
    Wh = (d + 3) // 4
    assert B.sylvie_wire_row_words_bits(d, 16) == Wh
    wire = torch.full((n * Wh + 3,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_bbit_fwd(dev(x), ld, d, dev(idx), 0, n, 16, 0, 0, wire)
    torch.cuda.synchronize()
    ref = oracle.convert_fp16(x, d, n, idx=idx)
    gw = wire.cpu().numpy()
    assert np.array_equal(gw[: n * Wh].view(np.uint16).reshape(n, 4 * Wh), ref)
    assert (gw[n * Wh:] == -1).all()
    # contiguous block
    wire2 = torch.full((100 * Wh,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_bbit_bwd(dev(x), ld, d, None, 50, 100, 16, 0, 0, wire2)
    ref2 = oracle.convert_fp16(x, d, 100, row_offset=50)
    assert np.array_equal(wire2.cpu().numpy().view(np.uint16).reshape(100, 4 * Wh), ref2)
    # recover, forward
    for ldo, off in ((d, 0), (d + 4, 9), (d + 1, 2)):
        o_ref = rng.standard_normal((n + 12, ldo)).astype(np.float32)
        out = dev(o_ref)
        oracle.recover_fp16_fwd(ref, d, o_ref, off)
        B.sylvie_dequantize_bbit_fwd(wire, n, d, 16, out, ldo, off)
        torch.cuda.synchronize()
        assert np.array_equal(bits32(out.cpu().numpy()), bits32(o_ref)), (ldo, off)
    # recover, backward accumulate
    n_dst = 200
    dst = rng.integers(0, n_dst - 20, n).astype(np.int32)
    dst[:30] = 5
    ldj = d + (3 if d % 2 else 4)
    J = rng.standard_normal((n_dst, ldj)).astype(np.float32)
    Jg = dev(J)
    oracle.recover_fp16_bwd(ref, d, J, dst)
    sp_, sr, di = GE.scatter_segments(dev(dst))
    B.sylvie_dequantize_bbit_bwd(wire, n, d, 16, Jg, ldj, sp_, sr, int(di.numel()), di)
    torch.cuda.synchronize()
    assert np.array_equal(bits32(Jg.cpu().numpy()), bits32(J))


def _join_bits(pk, sc, zp):
    n, Wb = pk.shape
    w = np.empty((n, Wb + 1), np.uint64)
    w[:, :Wb] = pk
    w[:, Wb] = (zp.view(np.uint32).astype(np.uint64) << np.uint64(32)) | sc.view(np.uint32).astype(np.uint64)
    return w.view(np.int64)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("d", [4, 64, 100, 128, 256, 300, 512, 1024])
@pytest.mark.parametrize("cfg,n_nodes,model", [("stress", 30_000, "gcn"), ("co_purchase", 20_000, "sage")])
def test_aggregate_from_bbit_wire_parity(oracle, bits, d, cfg, n_nodes, model):
    """Forward aggregation reading b-bit wire rows (Eq. 5 with B = 2^b - 1 applied to each gathered
    element): against the oracle's dequantize followed by its aggregate, to the float tolerance,
    and against the GPU's own two-step path."""
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    from test_gpu_ops import _operator, close
    p, (rp, cl, w) = _operator(oracle, cfg, n_nodes, model)
    n_loc = p.n_in + p.n_halo
    rng = np.random.default_rng(d + bits)
    X = make_rows(rng, n_loc, d, "heavy")
    pk, sc, zp = oracle.quantize_bbit(X, d, p.n_halo, bits, 77, 2, row_offset=p.n_in)
    Xo = X.copy()
    oracle.dequantize_bbit_fwd(pk, sc, zp, d, bits, Xo, p.n_in)
    Z, S = oracle.aggregate_fwd(rp, cl, w, Xo, d, want_S=True)
    rpd, cld, wd = dev(rp), dev(cl), dev(w)
    Xin = dev(X[: p.n_in])
    wired = dev(_join_bits(pk, sc, zp))
    for chunk in (0, 128):
        kw = {}
        if chunk:
            lr, lp, nt = GE.long_row_plan(rpd, chunk)
            kw = dict(chunk=chunk, long_rows=lr, long_ptr=lp, n_long=int(lr.numel()), n_tasks=nt,
                      workspace=torch.empty(max(1, nt) * d, device=DEV))
        Y = torch.full((p.n_in, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_fwd_wire_bbit(rpd, cld, wd, None, None, p.n_in, Xin, d, d, bits, p.n_in,
                                             wired, p.n_halo, Y, d, **kw)
        Xfull = dev(X)
        B.sylvie_dequantize_bbit_fwd(wired, p.n_halo, d, bits, Xfull, d, p.n_in)
        Y2 = torch.full((p.n_in, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_fwd(rpd, cld, wd, None, None, p.n_in, Xfull, d, d, Y2, d, **kw)
        torch.cuda.synchronize()
        close(Y.cpu().numpy(), Z, S, ("bbit wire", bits, chunk))
        close(Y.cpu().numpy(), Y2.cpu().numpy().astype(np.float64), S, ("bbit wire vs two-step", bits, chunk))


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("d", [4, 64, 100, 256, 600])
@pytest.mark.parametrize("cfg,n_nodes,model", [("stress", 30_000, "gcn"), ("co_purchase", 20_000, "sage")])
def test_backward_epilogues_bbit_equal_two_step(oracle, bits, d, cfg, n_nodes, model):
    """aggregate_csr_bwd_quantize_bbit / _integrate_bbit against the GPU's own aggregate_csr_bwd +
    quantize_bbit_bwd + dequantize_bbit_bwd, bit for bit; the wire is also recomputed by the
    oracle from the GPU's float rows."""
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    from test_gpu_ops import _operator
    p, (rp, cl, w) = _operator(oracle, cfg, n_nodes, model)
    n_loc = p.n_in + p.n_halo
    rng = np.random.default_rng(d + 3 + bits)
    dZ = dev(make_rows(rng, p.n_in, d, "heavy"))
    add = dev(make_rows(rng, p.n_in, d, "normal"))
    mirror = dev(rng.integers(0, p.n_in, p.n_halo).astype(np.int32))
    rpT, clT, wT = GE.transpose_csr(dev(rp), dev(cl), dev(w), n_loc)
    W1 = (d * bits + 63) // 64 + 1
    seed, sid, chunk = 4242 + d, 5, 128
    lr, lp, nt = GE.long_row_plan(rpT, chunk)
    ws = torch.empty(max(1, nt) * d, device=DEV)
    G = torch.full((n_loc, d), float("nan"), device=DEV)
    B.sylvie_aggregate_csr_bwd(rpT, clT, wT, None, None, n_loc, dZ, d, d, G, d, addend=add, ld_addend=d,
                               addend_rows=p.n_in, chunk=chunk, long_rows=lr, long_ptr=lp,
                               n_long=int(lr.numel()), n_tasks=nt, workspace=ws)
    wire_ref = torch.full((p.n_halo * W1,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_bbit_bwd(G, d, d, None, p.n_in, p.n_halo, bits, seed, sid, wire_ref)
    sp_, sr, di = GE.scatter_segments(mirror)
    Gpre = G.clone()
    B.sylvie_dequantize_bbit_bwd(wire_ref, p.n_halo, d, bits, G, d, sp_, sr, int(di.numel()), di)
    lrh, lph, nth = GE.long_row_plan(rpT, chunk, p.n_in, n_loc)
    wire = torch.full((p.n_halo * W1,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_aggregate_csr_bwd_quantize_bbit(rpT, clT, wT, None, None, p.n_in, p.n_halo, dZ, d, d, bits, seed,
                                             sid, wire, chunk=chunk, long_rows=lrh, long_ptr=lph,
                                             n_long=int(lrh.numel()), n_tasks=nth, workspace=ws)
    lri, lpi, nti = GE.long_row_plan(rpT, chunk, 0, p.n_in)
    sp2, sr2 = GE.scatter_segments_dense(mirror, p.n_in)
    J = torch.full((p.n_in, d), float("nan"), device=DEV)
    B.sylvie_aggregate_csr_bwd_integrate_bbit(rpT, clT, wT, None, None, 0, p.n_in, dZ, d, d, bits, J, d, add, d,
                                              p.n_in, wire, p.n_halo, sp2, sr2, chunk=chunk,
                                              long_rows=lri, long_ptr=lpi, n_long=int(lri.numel()),
                                              n_tasks=nti, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(wire, wire_ref)
    assert np.array_equal(bits32(J.cpu().numpy()), bits32(G[: p.n_in].cpu().numpy()))
    ref = oracle.quantize_bbit(Gpre.cpu().numpy(), d, p.n_halo, bits, seed, sid, row_offset=p.n_in)
    pk, sc, zp = split_wire_bits(wire.cpu().numpy(), p.n_halo, d, bits)
    assert np.array_equal(pk, ref[0]) and np.array_equal(bits32(sc), bits32(ref[1])) and \
        np.array_equal(bits32(zp), bits32(ref[2]))


def test_bbit_fused_calls_need_aligned_rows(oracle):
    """Widths that are not a multiple of 4 are refused with a status, nothing is enqueued."""
    from paper_2303_01277_amd import binding as B
    t = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=DEV)
    rp = torch.tensor([0, 1], dtype=torch.int64, device=DEV)
    cl = torch.tensor([1], dtype=torch.int32, device=DEV)
    with pytest.raises(B.SylvieError, match="not implemented"):
        B.sylvie_aggregate_csr_fwd_wire_bbit(rp, cl, None, None, None, 1, t(1, 6), 6, 6, 4, 1,
                                             t(8, dt=torch.int64), 1, t(1, 6), 6)
    with pytest.raises(B.SylvieError, match="bits"):
        B.sylvie_aggregate_csr_fwd_wire_bbit(rp, cl, None, None, None, 1, t(1, 8), 8, 8, 3, 1,
                                             t(8, dt=torch.int64), 1, t(1, 8), 8)


@pytest.mark.parametrize("d", [1, 3, 64, 100, 255, 256, 602])
def test_full_precision_wire(d):
    """bits = 32, the vanilla exchange of the bit-width study: the rows themselves travel.  Sending
    is a row gather, receiving a copy, the backward direction the ordered accumulate; checked
    against plain indexing and numpy's unbuffered in-order add."""
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    rng = np.random.default_rng(d)
    n_src, n, n_dst = 300, 517, 200
    ld = d + (5 if d % 2 else 0)
    x = make_rows(rng, n_src, ld, "heavy")
    idx = rng.integers(0, n_src, n).astype(np.int32)
    W = B.sylvie_wire_row_words_bits(d, 32)
    assert W == (d + 1) // 2
    wire = torch.full((n * W + 3,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_bbit_fwd(dev(x), ld, d, dev(idx), 0, n, 32, 0, 0, wire)
    torch.cuda.synchronize()
    gw = wire.cpu().numpy()
    rows = gw[: n * W].view(np.float32).reshape(n, 2 * W)
    assert np.array_equal(bits32(rows[:, :d]), bits32(x[idx][:, :d])) and (gw[n * W:] == -1).all()
    assert not rows[:, d:].any()
    out = torch.full((n + 7, ld), float("nan"), device=DEV)
    B.sylvie_dequantize_bbit_fwd(wire, n, d, 32, out, ld, 5)
    J = rng.standard_normal((n_dst, ld)).astype(np.float32)
    Jg = dev(J)
    dst = rng.integers(0, n_dst - 20, n).astype(np.int32)
    dst[:30] = 11
    sp_, sr, di = GE.scatter_segments(dev(dst))
    B.sylvie_dequantize_bbit_bwd(wire, n, d, 32, Jg, ld, sp_, sr, int(di.numel()), di)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    assert np.array_equal(bits32(o[5: 5 + n, :d]), bits32(x[idx][:, :d])) and np.isnan(o[:5]).all()
    ref = J.copy()
    np.add.at(ref[:, :d], dst, x[idx][:, :d])
    assert np.array_equal(bits32(Jg.cpu().numpy()), bits32(ref))


@pytest.mark.parametrize("d", [4, 64, 100, 256, 600])
@pytest.mark.parametrize("cfg,n_nodes,model", [("stress", 30_000, "gcn"), ("co_purchase", 20_000, "sage")])
def test_fused_half_precision_wire(oracle, d, cfg, n_nodes, model):
    """bits = 16 of the three fused aggregation calls (the bit-width study's half-precision point):
    the forward aggregation that reads binary16 halo rows against the oracle's recover + aggregate
    and the GPU's two-step path; the backward epilogues against aggregate_csr_bwd + the stand-alone
    conversion / accumulate bit for bit, the wire also against the oracle's conversion."""
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    from test_gpu_ops import _operator, close
    p, (rp, cl, w) = _operator(oracle, cfg, n_nodes, model)
    n_loc = p.n_in + p.n_halo
    rng = np.random.default_rng(d + 16)
    X = make_rows(rng, n_loc, d, "heavy")
    Wh = (d + 3) // 4
    half = oracle.convert_fp16(X, d, p.n_halo, row_offset=p.n_in)
    Xo = X.copy()
    oracle.recover_fp16_fwd(half, d, Xo, p.n_in)
    Z, S = oracle.aggregate_fwd(rp, cl, w, Xo, d, want_S=True)
    rpd, cld, wd, Xfull = dev(rp), dev(cl), dev(w), dev(X)
    wired = torch.full((p.n_halo * Wh,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_bbit_fwd(Xfull, d, d, None, p.n_in, p.n_halo, 16, 0, 0, wired)
    for chunk in (0, 128):
        kw = {}
        if chunk:
            lr, lp, nt = GE.long_row_plan(rpd, chunk)
            kw = dict(chunk=chunk, long_rows=lr, long_ptr=lp, n_long=int(lr.numel()), n_tasks=nt,
                      workspace=torch.empty(max(1, nt) * d, device=DEV))
        Y = torch.full((p.n_in, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_fwd_wire_bbit(rpd, cld, wd, None, None, p.n_in, Xfull, d, d, 16, p.n_in, wired,
                                             p.n_halo, Y, d, **kw)
        X2 = Xfull.clone()
        B.sylvie_dequantize_bbit_fwd(wired, p.n_halo, d, 16, X2, d, p.n_in)
        Y2 = torch.full((p.n_in, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_fwd(rpd, cld, wd, None, None, p.n_in, X2, d, d, Y2, d, **kw)
        torch.cuda.synchronize()
        close(Y.cpu().numpy(), Z, S, ("half wire", chunk))
        close(Y.cpu().numpy(), Y2.cpu().numpy().astype(np.float64), S, ("half wire vs two-step", chunk))
    # backward epilogues
    dZ = dev(make_rows(rng, p.n_in, d, "heavy"))
    add = dev(make_rows(rng, p.n_in, d, "normal"))
    mirror = dev(rng.integers(0, p.n_in, p.n_halo).astype(np.int32))
    rpT, clT, wT = GE.transpose_csr(rpd, cld, wd, n_loc)
    chunk = 128
    lr, lp, nt = GE.long_row_plan(rpT, chunk)
    ws = torch.empty(max(1, nt) * d, device=DEV)
    G = torch.full((n_loc, d), float("nan"), device=DEV)
    B.sylvie_aggregate_csr_bwd(rpT, clT, wT, None, None, n_loc, dZ, d, d, G, d, addend=add, ld_addend=d,
                               addend_rows=p.n_in, chunk=chunk, long_rows=lr, long_ptr=lp,
                               n_long=int(lr.numel()), n_tasks=nt, workspace=ws)
    wire_ref = torch.full((p.n_halo * Wh,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_bbit_bwd(G, d, d, None, p.n_in, p.n_halo, 16, 0, 0, wire_ref)
    sp_, sr, di = GE.scatter_segments(mirror)
    Gpre = G.clone()
    B.sylvie_dequantize_bbit_bwd(wire_ref, p.n_halo, d, 16, G, d, sp_, sr, int(di.numel()), di)
    lrh, lph, nth = GE.long_row_plan(rpT, chunk, p.n_in, n_loc)
    wire = torch.full((p.n_halo * Wh,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_aggregate_csr_bwd_quantize_bbit(rpT, clT, wT, None, None, p.n_in, p.n_halo, dZ, d, d, 16, 0, 0, wire,
                                             chunk=chunk, long_rows=lrh, long_ptr=lph, n_long=int(lrh.numel()),
                                             n_tasks=nth, workspace=ws)
    lri, lpi, nti = GE.long_row_plan(rpT, chunk, 0, p.n_in)
    sp2, sr2 = GE.scatter_segments_dense(mirror, p.n_in)
    J = torch.full((p.n_in, d), float("nan"), device=DEV)
    B.sylvie_aggregate_csr_bwd_integrate_bbit(rpT, clT, wT, None, None, 0, p.n_in, dZ, d, d, 16, J, d, add, d,
                                              p.n_in, wire, p.n_halo, sp2, sr2, chunk=chunk, long_rows=lri,
                                              long_ptr=lpi, n_long=int(lri.numel()), n_tasks=nti, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(wire, wire_ref)
    assert np.array_equal(bits32(J.cpu().numpy()), bits32(G[: p.n_in].cpu().numpy()))
    ref = oracle.convert_fp16(Gpre.cpu().numpy(), d, p.n_halo, row_offset=p.n_in)
    assert np.array_equal(wire.cpu().numpy().view(np.uint16).reshape(p.n_halo, 4 * Wh), ref)
