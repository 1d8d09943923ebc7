"""GPU parity, op by op: every entry point of the C ABI against the CPU oracle on
the same seeded inputs.  Bit-exact for packed words, scale, zero, dequantised rows and
the backward accumulate; |gpu - ref| <= 1e-5 * max(|ref|, S) for the float sums, S the
oracle's sum of |terms| (aggregate, transform)."""
import numpy as np
import pytest
import torch

from synth import CONFIGS, build_workload, scaled
from util import join_wire, split_wire

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-5


def bits32(a):
    return np.ascontiguousarray(a).view(np.uint32)


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def close(got, ref, S, what):
    got = got.astype(np.float64)
    err = np.abs(got - ref.astype(np.float64))
    bound = TOL * np.maximum(np.abs(ref), S).astype(np.float64)
    bad = err > bound
    assert not bad.any(), (what, int(bad.sum()), float((err / np.maximum(bound, 1e-300)).max()))


def make_rows(rng, n, ld, kind):
    x = rng.standard_normal((n, ld)).astype(np.float32)
    if kind == "heavy":
        x *= np.exp(2 * rng.standard_normal((n, 1))).astype(np.float32)
    if kind == "relu":
        x = np.maximum(x, 0)
        x[::7] = 0.0                      # all-zero rows
    if kind == "edge" and n >= 8:
        x[0] = 3.25                       # constant
        x[1] = -0.0                       # negative zeros
        x[2] = np.float32(1e-38) * rng.integers(0, 5, ld).astype(np.float32)   # subnormal range
        x[3] = np.float32(2.0 ** -110) * rng.standard_normal(ld).astype(np.float32)  # tiny scale
        x[4] = np.float32(1e37) * rng.uniform(-1, 1, ld).astype(np.float32)    # huge
        x[5, :] = 0.0
        x[5, ld // 2] = -0.0
        x[6] = np.where(rng.integers(0, 2, ld) > 0, 1.0, -1.0).astype(np.float32)
    return x


def run_quantize(B, oracle, x, d, n, idx, row_offset, seed, stream, fn):
    W1 = (d + 63) // 64 + 1
    xs = dev(x)
    wire = torch.full((n * W1 + 3,), -1, dtype=torch.int64, device=DEV)
    fn(xs, x.shape[1], d, None if idx is None else dev(idx), row_offset, n, seed, stream, wire)
    torch.cuda.synchronize()
    ref = oracle.quantize_1bit(x, d, n, seed, stream, idx=idx, row_offset=row_offset)
    gw = wire.cpu().numpy()
    pk, sc, zp = split_wire(gw, n, d)
    assert np.array_equal(pk, ref[0]), "packed words"
    assert np.array_equal(bits32(sc), bits32(ref[1])), "scale"
    assert np.array_equal(bits32(zp), bits32(ref[2])), "zero"
    assert (gw[n * W1:] == -1).all()                            # nothing written past the end
    return wire, ref


@pytest.mark.parametrize("d", [1, 2, 3, 63, 64, 65, 100, 128, 129, 256, 300, 602, 640, 1024, 1100])
@pytest.mark.parametrize("kind", ["normal", "edge", "relu", "heavy"])
def test_quantize_parity(oracle, d, kind):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(d * 31 + len(kind))
    n_src, n = 700, 1003                                        # several tiles + ragged tail
    ld = d + (5 if d % 2 else 0)
    x = make_rows(rng, n_src, ld, kind)
    idx = rng.integers(0, n_src, n).astype(np.int32)            # gather with duplicates
    run_quantize(B, oracle, x, d, n, idx, 0, 0xABCDEF0123456789 + d, 2 * 3 + 0,
                 B.sylvie_quantize_1bit_fwd)
    # contiguous block (the backward convention): rows [row_offset, row_offset + n)
    run_quantize(B, oracle, x, d, 333, None, 300, 12345 + d, 2 * 3 + 1,
                 B.sylvie_quantize_1bit_bwd)


def test_quantize_tiny_counts(oracle):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(3)
    x = make_rows(rng, 40, 256, "normal")
    for n in (1, 2, 3, 4, 5, 15, 16, 17):
        run_quantize(B, oracle, x, 256, n, None, 7, 99, 1, B.sylvie_quantize_1bit_fwd)
    # n = 0: nothing is written, nothing fails
    p = torch.zeros(8, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_1bit_fwd(dev(x), 256, 256, None, 0, 0, 1, 1, p)


@pytest.mark.parametrize("d", [1, 2, 3, 64, 65, 100, 128, 256, 602, 1100])
def test_dequantize_fwd_parity(oracle, d):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(d)
    n = 517
    x = make_rows(rng, n, d, "edge")
    pk, sc, zp = oracle.quantize_1bit(x, d, n, 5, 0)
    for ld, off in ((d, 0), (d + 4, 11), (d + 1, 3)):
        ref = rng.standard_normal((n + 20, ld)).astype(np.float32)
        out = dev(ref)
        oracle.dequantize_1bit_fwd(pk, sc, zp, d, ref, off)
        B.sylvie_dequantize_1bit_fwd(dev(join_wire(pk, sc, zp)), n, d, out, ld, off)
        torch.cuda.synchronize()
        assert np.array_equal(bits32(out.cpu().numpy()), bits32(ref)), (ld, off)


@pytest.mark.parametrize("d", [1, 3, 64, 100, 256, 602])
def test_dequantize_bwd_parity(oracle, d):
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    rng = np.random.default_rng(d + 1)
    n, n_dst = 900, 400
    g = make_rows(rng, n, d, "heavy")
    pk, sc, zp = oracle.quantize_1bit(g, d, n, 8, 3)
    dst = rng.integers(0, n_dst - 50, n).astype(np.int32)       # duplicates; rows >= 350 untouched
    dst[:40] = 17                                               # one long segment
    ld = d + (3 if d % 2 else 4)
    J = rng.standard_normal((n_dst, ld)).astype(np.float32)
    Jg = dev(J)
    oracle.dequantize_1bit_bwd(pk, sc, zp, d, J, dst)
    sp_, sr, di = GE.scatter_segments(dev(dst))
    B.sylvie_dequantize_1bit_bwd(dev(join_wire(pk, sc, zp)), n, d, Jg, ld, sp_, sr,
                                 int(di.numel()), di)
    torch.cuda.synchronize()
    assert np.array_equal(bits32(Jg.cpu().numpy()), bits32(J))


def _operator(oracle, cfg, n_nodes, model):
    wl = build_workload(scaled(CONFIGS[cfg], n_nodes))
    p = wl.parts[0]
    rp, cl, dg = p.rowptr.numpy(), p.col.numpy(), p.deg.numpy()
    if model == "gcn":
        return p, oracle.gcn_operator(rp, cl, dg, p.n_in)
    return p, (rp, cl, oracle.mean_weights(rp, p.n_in))


@pytest.mark.parametrize("d", [7, 64, 100, 128, 256, 602])
@pytest.mark.parametrize("cfg,n_nodes,model", [("stress", 40_000, "gcn"),
                                               ("co_purchase", 30_000, "sage")])
def test_aggregate_parity(oracle, d, cfg, n_nodes, model):
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    p, (rp, cl, w) = _operator(oracle, cfg, n_nodes, model)
    n_loc = p.n_in + p.n_halo
    rng = np.random.default_rng(d)
    X = make_rows(rng, n_loc, d, "heavy")
    Z, S = oracle.aggregate_fwd(rp, cl, w, X, d, want_S=True)
    rpd, cld, wd, Xd = dev(rp), dev(cl), dev(w), dev(X)
    for chunk in (0, 64, 1024):
        Y = torch.full((p.n_in, d), float("nan"), device=DEV)
        if chunk:
            lr, lp, nt = GE.long_row_plan(rpd, chunk)
            ws = torch.empty(max(1, nt) * d, device=DEV)
            B.sylvie_aggregate_csr_fwd(rpd, cld, wd, None, None, p.n_in, Xd, d, d, Y, d,
                                       chunk=chunk, long_rows=lr, long_ptr=lp,
                                       n_long=int(lr.numel()), n_tasks=nt, workspace=ws)
        else:
            B.sylvie_aggregate_csr_fwd(rpd, cld, wd, None, None, p.n_in, Xd, d, d, Y, d)
        torch.cuda.synchronize()
        close(Y.cpu().numpy(), Z, S, ("fwd", chunk))
    # transpose product on the transposed CSR, against the oracle's scatter
    dZ = make_rows(rng, p.n_in, d, "normal")
    dX, Sb = oracle.aggregate_bwd(rp, cl, w, n_loc, dZ, d, want_S=True)
    rpT, clT, wT = GE.transpose_csr(rpd, cld, wd, n_loc)
    lr, lp, nt = GE.long_row_plan(rpT, 128)
    ws = torch.empty(max(1, nt) * d, device=DEV)
    add = make_rows(rng, p.n_in, d, "normal")
    for use_add in (False, True):
        Y = torch.full((n_loc, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_bwd(rpT, clT, wT, None, None, n_loc, dev(dZ), d, d, Y, d,
                                   addend=dev(add) if use_add else None, ld_addend=d,
                                   addend_rows=p.n_in, chunk=128, long_rows=lr, long_ptr=lp,
                                   n_long=int(lr.numel()), n_tasks=nt, workspace=ws)
        torch.cuda.synchronize()
        ref, Sr = dX.astype(np.float64), Sb.copy()
        if use_add:
            ref = ref.copy()
            ref[: p.n_in] += add
            Sr[: p.n_in] += np.abs(add)
        close(Y.cpu().numpy(), ref, Sr, ("bwd", use_add))


def test_aggregate_scales_and_unit_weights(oracle):
    """w = NULL with row/col scales reproduces the explicit-weight GCN operator."""
    from paper_2303_01277_amd import binding as B
    p, (rp, cl, w) = _operator(oracle, "citation", 20_000, "gcn")
    n_loc = p.n_in + p.n_halo
    d = 128
    rng = np.random.default_rng(0)
    X = make_rows(rng, n_loc, d, "normal")
    Z, S = oracle.aggregate_fwd(rp, cl, w, X, d, want_S=True)
    dinv = (1.0 / np.sqrt(p.deg.numpy().astype(np.float64) + 1)).astype(np.float32)
    Y = torch.empty((p.n_in, d), device=DEV)
    B.sylvie_aggregate_csr_fwd(dev(rp), dev(cl), None, dev(dinv[: p.n_in]), dev(dinv), p.n_in,
                               dev(X), d, d, Y, d)
    torch.cuda.synchronize()
    close(Y.cpu().numpy(), Z, S * (1 + 1e-6), "scales")


@pytest.mark.parametrize("n,k1,k2,h", [(1000, 64, 0, 64), (777, 256, 0, 256), (300, 602, 0, 256),
                                        (515, 100, 100, 128), (129, 128, 0, 40), (64, 20, 0, 7),
                                        (515, 96, 32, 128), (300, 64, 0, 384), (2000, 256, 256, 256),
                                        (131, 128, 128, 200), (1, 16, 0, 4), (4100, 16, 16, 16)])
def test_transform_parity(oracle, n, k1, k2, h):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(n + k1)
    A1 = make_rows(rng, n, k1, "relu")
    A2 = make_rows(rng, n, k2, "normal") if k2 else None
    W = (rng.standard_normal((k1 + k2, h)) / np.sqrt(k1 + k2)).astype(np.float32)
    J = make_rows(rng, n, h, "normal")
    for relu in (True, False):
        Href, S = oracle.transform_fwd(A1, W, relu, A2=A2, want_S=True)
        Hg = torch.full((n, h), float("nan"), device=DEV)
        B.sylvie_transform_fwd(dev(A1), k1, k1, None if A2 is None else dev(A2), k2, k2, dev(W), h,
                               n, relu, Hg, h)
        torch.cuda.synchronize()
        Hgn = Hg.cpu().numpy()
        close(Hgn, Href, S, ("H", relu))
        # backward is teacher-forced with the GPU's own forward output as the mask
        r = oracle.transform_bwd(A1, W, relu, Hgn, J, A2=A2, want_S=True)
        G = torch.full((k1 + k2, h), float("nan"), device=DEV)
        dA1 = torch.full((n, k1), float("nan"), device=DEV)
        dA2 = torch.full((n, k2), float("nan"), device=DEV) if k2 else None
        ws = torch.empty(B.sylvie_transform_bwd_workspace_bytes(k1, k2, h, n) // 4, device=DEV)
        B.sylvie_transform_bwd(dev(A1), k1, k1, None if A2 is None else dev(A2), k2, k2, dev(W), h,
                               n, relu, Hg, h, dev(J), h, G, dA1, k1, dA2, k2, ws)
        torch.cuda.synchronize()
        close(G.cpu().numpy(), r["G"], r["SG"], ("G", relu))
        close(dA1.cpu().numpy(), r["dA1"], r["SdA1"], ("dA1", relu))
        if k2:
            close(dA2.cpu().numpy(), r["dA2"], r["SdA2"], ("dA2", relu))


@pytest.mark.parametrize("n,k1,k2,h", [(700, 128, 0, 256), (300, 64, 64, 144), (257, 100, 0, 36)])
def test_transform_strided(oracle, n, k1, k2, h):
    """Operands and results that are column blocks of wider row-major buffers (leading
    dimension > width); whatever lies outside the blocks must stay untouched."""
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(n + h)
    A1 = make_rows(rng, n, k1, "relu")
    A2 = make_rows(rng, n, k2, "normal") if k2 else None
    W = (rng.standard_normal((k1 + k2, h)) / np.sqrt(k1 + k2)).astype(np.float32)
    J = make_rows(rng, n, h, "normal")

    def wide(a, pad):
        """device buffer [rows, width + pad] holding a in its first columns, 7.0 elsewhere"""
        buf = torch.full((a.shape[0], a.shape[1] + pad), 7.0, device=DEV)
        buf[:, : a.shape[1]] = dev(a)
        return buf

    for relu in (True, False):
        Href, S = oracle.transform_fwd(A1, W, relu, A2=A2, want_S=True)
        a1 = wide(A1, 8)
        a2 = wide(A2, 4) if k2 else None
        Hg = torch.full((n, h + 12), 7.0, device=DEV)
        B.sylvie_transform_fwd(a1, k1 + 8, k1, a2, k2 + 4, k2, dev(W), h, n, relu, Hg, h + 12)
        torch.cuda.synchronize()
        Hgn = np.ascontiguousarray(Hg[:, :h].cpu().numpy())
        close(Hgn, Href, S, ("H", relu))
        assert bool((Hg[:, h:] == 7.0).all())
        r = oracle.transform_bwd(A1, W, relu, Hgn, J, A2=A2, want_S=True)
        G = torch.full((k1 + k2, h), float("nan"), device=DEV)
        dA1 = torch.full((n, k1 + 4), 7.0, device=DEV)
        dA2 = torch.full((n, k2 + 8), 7.0, device=DEV) if k2 else None
        jw = wide(J, 4)
        ws = torch.empty(B.sylvie_transform_bwd_workspace_bytes(k1, k2, h, n) // 4, device=DEV)
        B.sylvie_transform_bwd(a1, k1 + 8, k1, a2, k2 + 4, k2, dev(W), h, n, relu, Hg, h + 12, jw, h + 4,
                               G, dA1, k1 + 4, dA2, k2 + 8, ws)
        torch.cuda.synchronize()
        close(G.cpu().numpy(), r["G"], r["SG"], ("G", relu))
        close(np.ascontiguousarray(dA1[:, :k1].cpu().numpy()), r["dA1"], r["SdA1"], ("dA1", relu))
        assert bool((dA1[:, k1:] == 7.0).all())
        if k2:
            close(np.ascontiguousarray(dA2[:, :k2].cpu().numpy()), r["dA2"], r["SdA2"], ("dA2", relu))
            assert bool((dA2[:, k2:] == 7.0).all())


@pytest.mark.parametrize("d", [2, 7, 64, 65, 100, 128, 129, 160, 256, 300, 301, 602, 1024])
@pytest.mark.parametrize("cfg,n_nodes,model", [("stress", 40_000, "gcn"),
                                               ("co_purchase", 30_000, "sage")])
def test_aggregate_from_wire_parity(oracle, d, cfg, n_nodes, model):
    """Fused dequantize + aggregate: against the oracle's dequantize followed by its
    aggregate, and against the GPU's own two-step path (same terms; wide rows sum their
    wire entries in accumulators of their own, so the order of the additions differs)."""
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    p, (rp, cl, w) = _operator(oracle, cfg, n_nodes, model)
    n_loc = p.n_in + p.n_halo
    rng = np.random.default_rng(d + 7)
    X = make_rows(rng, n_loc, d, "heavy")
    pk, sc, zp = oracle.quantize_1bit(X, d, p.n_halo, 77, 2, row_offset=p.n_in)
    Xo = X.copy()
    oracle.dequantize_1bit_fwd(pk, sc, zp, d, Xo, p.n_in)       # halo block := recovered rows
    Z, S = oracle.aggregate_fwd(rp, cl, w, Xo, d, want_S=True)
    rpd, cld, wd = dev(rp), dev(cl), dev(w)
    Xin = dev(X[: p.n_in])
    wired = dev(join_wire(pk, sc, zp))
    for chunk in (0, 128):
        kw = {}
        if chunk:
            lr, lp, nt = GE.long_row_plan(rpd, chunk)
            kw = dict(chunk=chunk, long_rows=lr, long_ptr=lp, n_long=int(lr.numel()), n_tasks=nt,
                      workspace=torch.empty(max(1, nt) * d, device=DEV))
        Y = torch.full((p.n_in, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_fwd_wire(rpd, cld, wd, None, None, p.n_in, Xin, d, d, p.n_in, wired,
                                        p.n_halo, Y, d, **kw)
        Xfull = dev(X)
        B.sylvie_dequantize_1bit_fwd(wired, p.n_halo, d, Xfull, d, p.n_in)
        Y2 = torch.full((p.n_in, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_fwd(rpd, cld, wd, None, None, p.n_in, Xfull, d, d, Y2, d, **kw)
        torch.cuda.synchronize()
        close(Y.cpu().numpy(), Z, S, ("wire", chunk))
        close(Y.cpu().numpy(), Y2.cpu().numpy().astype(np.float64), S, ("wire vs two-step", chunk))


@pytest.mark.parametrize("d", [2, 7, 64, 100, 256, 602])
@pytest.mark.parametrize("cfg,n_nodes,model", [("stress", 30_000, "gcn"), ("co_purchase", 20_000, "sage")])
def test_backward_epilogues_equal_two_step(oracle, d, cfg, n_nodes, model):
    """aggregate_csr_bwd_quantize / _integrate against the GPU's own aggregate_csr_bwd +
    quantize_1bit_bwd + dequantize_1bit_bwd (bit for bit), whose pieces are tied to the
    oracle above; the wire is also recomputed by the oracle from the GPU's float rows."""
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    p, (rp, cl, w) = _operator(oracle, cfg, n_nodes, model)
    n_loc = p.n_in + p.n_halo
    rng = np.random.default_rng(d + 3)
    dZ = dev(make_rows(rng, p.n_in, d, "heavy"))
    add = dev(make_rows(rng, p.n_in, d, "normal"))
    mirror = dev(rng.integers(0, p.n_in, p.n_halo).astype(np.int32))
    rpT, clT, wT = GE.transpose_csr(dev(rp), dev(cl), dev(w), n_loc)
    W1 = (d + 63) // 64 + 1
    seed, sid, chunk = 4242 + d, 5, 128
    # two-step reference on the GPU
    lr, lp, nt = GE.long_row_plan(rpT, chunk)
    ws = torch.empty(max(1, nt) * d, device=DEV)
    G = torch.full((n_loc, d), float("nan"), device=DEV)
    B.sylvie_aggregate_csr_bwd(rpT, clT, wT, None, None, n_loc, dZ, d, d, G, d, addend=add,
                               ld_addend=d, addend_rows=p.n_in, chunk=chunk, long_rows=lr,
                               long_ptr=lp, n_long=int(lr.numel()), n_tasks=nt, workspace=ws)
    wire_ref = torch.full((p.n_halo * W1,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_quantize_1bit_bwd(G, d, d, None, p.n_in, p.n_halo, seed, sid, wire_ref)
    sp_, sr, di = GE.scatter_segments(mirror)
    Gpre = G.clone()
    B.sylvie_dequantize_1bit_bwd(wire_ref, p.n_halo, d, G, d, sp_, sr, int(di.numel()), di)
    # fused
    lrh, lph, nth = GE.long_row_plan(rpT, chunk, p.n_in, n_loc)
    wire = torch.full((p.n_halo * W1,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_aggregate_csr_bwd_quantize(rpT, clT, wT, None, None, p.n_in, p.n_halo, dZ, d, d, seed,
                                        sid, wire, chunk=chunk, long_rows=lrh, long_ptr=lph,
                                        n_long=int(lrh.numel()), n_tasks=nth, workspace=ws)
    lri, lpi, nti = GE.long_row_plan(rpT, chunk, 0, p.n_in)
    sp2, sr2 = GE.scatter_segments_dense(mirror, p.n_in)
    J = torch.full((p.n_in, d), float("nan"), device=DEV)
    B.sylvie_aggregate_csr_bwd_integrate(rpT, clT, wT, None, None, 0, p.n_in, dZ, d, d, J, d, add, d,
                                         p.n_in, wire, p.n_halo, sp2, sr2, chunk=chunk,
                                         long_rows=lri, long_ptr=lpi, n_long=int(lri.numel()),
                                         n_tasks=nti, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(wire, wire_ref)
    assert np.array_equal(bits32(J.cpu().numpy()), bits32(G[: p.n_in].cpu().numpy()))
    # the oracle's quantizer on the GPU's float halo rows gives the same wire
    ref = oracle.quantize_1bit(Gpre.cpu().numpy(), d, p.n_halo, seed, sid, row_offset=p.n_in)
    pk, sc, zp = split_wire(wire.cpu().numpy(), p.n_halo, d)
    assert np.array_equal(pk, ref[0]) and np.array_equal(bits32(sc), bits32(ref[1])) and \
        np.array_equal(bits32(zp), bits32(ref[2]))


def test_loop_without_halo(oracle):
    """A partition that owns the whole graph: no halo rows, empty wires, nothing to exchange."""
    from oracle import layers as OL
    from paper_2303_01277_amd.trainer import LayerLoop
    from util import np_c, to_partdata
    spec = scaled(CONFIGS["tiny"], 3000)
    spec = type(spec)(**{**spec.__dict__, "n_parts": 1, "dims": (64, 32, 16)})
    wl = build_workload(spec)
    pdata = to_partdata(wl)
    Wn = [np_c(w) for w in wl.W]
    OL.forward(pdata, "gcn", Wn, 1, "1bit")
    OL.backward(pdata, "gcn", Wn, 1, "1bit")
    p = wl.parts[0]
    assert p.n_halo == 0
    for f in ("rowptr", "col", "deg", "halo_gid", "halo_part", "halo_row"):
        setattr(p, f, getattr(p, f).to(DEV))
    for fused in (True, False):
        loop = LayerLoop([p], [p.halo_part], [p.halo_row], [wl.X[0].to(DEV)], [wl.J[0].to(DEV)],
                         [w.to(DEV) for w in wl.W], "gcn", spec.dims, chunk=64, fused=fused,
                         fused_bwd=fused)
        loop.forward(1)
        loop.backward(1)
        torch.cuda.synchronize()
        st = loop.parts[0]
        ref = pdata[0]
        assert np.abs(st.out.cpu().numpy() - ref.H[-1]).max() <= 2e-5 * np.abs(ref.H[-1]).max()
        assert np.abs(st.dHtil[1].cpu().numpy()[: p.n_in] - ref.Jin[1]).max() <= \
            2e-5 * np.abs(ref.Jin[1]).max()
        assert np.abs(st.G[1].cpu().numpy() - ref.G[1]).max() <= 2e-5 * np.abs(ref.G[1]).max()


@pytest.mark.parametrize("d", [64, 100, 256])
def test_row_order_changes_nothing(oracle, d):
    """A processing order (any permutation of the launch's rows) leaves every aggregation entry
    point's result bit for bit what it is in index order."""
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    p, (rp, cl, w) = _operator(oracle, "stress", 30_000, "gcn")
    n_loc = p.n_in + p.n_halo
    rng = np.random.default_rng(d + 11)
    X = make_rows(rng, n_loc, d, "heavy")
    pk, sc, zp = oracle.quantize_1bit(X, d, p.n_halo, 5, 2, row_offset=p.n_in)
    rpd, cld, wd = dev(rp), dev(cl), dev(w)
    wired = dev(join_wire(pk, sc, zp))
    Xin, Xfull = dev(X[: p.n_in]), dev(X)
    chunk = 128
    lr, lp, nt = GE.long_row_plan(rpd, chunk)
    kw = dict(chunk=chunk, long_rows=lr, long_ptr=lp, n_long=int(lr.numel()), n_tasks=nt,
              workspace=torch.empty(max(1, nt) * d, device=DEV))
    orders = [None, GE.rows_by_length(rpd), dev(rng.permutation(p.n_in).astype(np.int32))]
    outs = []
    for o in orders:
        Y1 = torch.full((p.n_in, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_fwd(rpd, cld, wd, None, None, p.n_in, Xfull, d, d, Y1, d, row_order=o, **kw)
        Y2 = torch.full((p.n_in, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_fwd_wire(rpd, cld, wd, None, None, p.n_in, Xin, d, d, p.n_in, wired,
                                        p.n_halo, Y2, d, row_order=o, **kw)
        outs.append((Y1, Y2))
    torch.cuda.synchronize()
    for Y1, Y2 in outs[1:]:
        assert torch.equal(Y1, outs[0][0]) and torch.equal(Y2, outs[0][1])
    # backward epilogues on a row range of the transposed operator
    rpT, clT, wT = GE.transpose_csr(rpd, cld, wd, n_loc)
    dZ = dev(make_rows(rng, p.n_in, d, "heavy"))
    mirror = dev(rng.integers(0, p.n_in, p.n_halo).astype(np.int32))
    sp_, sr = GE.scatter_segments_dense(mirror, p.n_in)
    W1 = (d + 63) // 64 + 1
    res = []
    for kind in ("index", "length", "random"):
        def order(r0, r1):
            if kind == "index":
                return None
            if kind == "length":
                return GE.rows_by_length(rpT, r0, r1)
            return dev(rng.permutation(r1 - r0).astype(np.int32))
        lrq, lpq, ntq = GE.long_row_plan(rpT, chunk, p.n_in, n_loc)
        wire = torch.full((p.n_halo * W1,), -1, dtype=torch.int64, device=DEV)
        B.sylvie_aggregate_csr_bwd_quantize(rpT, clT, wT, None, None, p.n_in, p.n_halo, dZ, d, d, 99, 7, wire,
                                            chunk=chunk, long_rows=lrq, long_ptr=lpq, n_long=int(lrq.numel()),
                                            n_tasks=ntq, workspace=torch.empty(max(1, ntq) * d, device=DEV),
                                            row_order=order(p.n_in, n_loc))
        lri, lpi, nti = GE.long_row_plan(rpT, chunk, 0, p.n_in)
        G = torch.full((p.n_in, d), float("nan"), device=DEV)
        B.sylvie_aggregate_csr_bwd_integrate(rpT, clT, wT, None, None, 0, p.n_in, dZ, d, d, G, d, None, 0, 0,
                                             wire, p.n_halo, sp_, sr, chunk=chunk, long_rows=lri, long_ptr=lpi,
                                             n_long=int(lri.numel()), n_tasks=nti,
                                             workspace=torch.empty(max(1, nti) * d, device=DEV),
                                             row_order=order(0, p.n_in))
        res.append((wire, G))
    torch.cuda.synchronize()
    for wire, G in res[1:]:
        assert torch.equal(wire, res[0][0]) and torch.equal(G, res[0][1])
