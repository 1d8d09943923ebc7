"""GPU parity of the attention-aggregator kernels (scores, edge softmax, sampled product,
softmax backward, row / column sums, rank-1 update, ReLU) against the CPU oracle, on operator
patterns with hub rows that are cut into several pieces."""
import numpy as np
import pytest
import torch

from test_gpu_ops import DEV, _operator, bits32, dev, make_rows

pytestmark = pytest.mark.gpu
TOL = 1e-5


def close(got, ref, S, what):
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = TOL * np.maximum(np.abs(ref), S).astype(np.float64) + 1e-30
    assert (err <= bound).all(), (what, int((err > bound).sum()), float((err / bound).max()))


def setup(oracle, n_nodes, chunk):
    from paper_2303_01277_amd import graph_engine as GE
    p, (rp, cl, w) = _operator(oracle, "stress", n_nodes, "gcn")
    rpd, cld = dev(rp), dev(cl)
    pieces = GE.piece_table(rpd, chunk)
    assert int(pieces[2][-1]) == pieces[1].numel() and int(pieces[0][-1]) == rp[-1]
    assert int((pieces[0][1:] - pieces[0][:-1]).max()) <= chunk and int((pieces[0][1:] - pieces[0][:-1]).min()) >= 1
    return p, rp, cl, rpd, cld, pieces


@pytest.mark.parametrize("chunk", [64, 1000])
@pytest.mark.parametrize("F", [1, 7, 64, 100, 256, 300])
def test_attention_kernels_parity(oracle, F, chunk):
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    p, rp, cl, rpd, cld, pieces = setup(oracle, 30_000, chunk)
    n_in, n_loc, nnz = p.n_in, p.n_in + p.n_halo, int(rp[-1])
    assert int((pieces[2][1:] - pieces[2][:-1]).max()) > 1 or chunk > 64      # hub rows were cut
    rng = np.random.default_rng(F + chunk)
    ld = F + (3 if F % 2 else 4)
    P = make_rows(rng, n_loc, ld, "normal")
    a_dst = (rng.standard_normal(F) / np.sqrt(F)).astype(np.float32)
    a_src = (rng.standard_normal(F) / np.sqrt(F)).astype(np.float32)
    Pd = dev(P)
    # scores
    s_dst_g = torch.empty(n_in, device=DEV); s_src_g = torch.empty(n_loc, device=DEV)
    B.sylvie_row_dot(Pd, ld, n_in, F, dev(a_dst), s_dst_g)
    B.sylvie_row_dot(Pd, ld, n_loc, F, dev(a_src), s_src_g)
    torch.cuda.synchronize()
    Pc = np.ascontiguousarray(P[:, :F])
    mag = np.abs(Pc.astype(np.float64)) @ np.abs(a_src.astype(np.float64))
    close(s_src_g.cpu().numpy(), oracle.row_dot(Pc, a_src), mag, "s_src")
    close(s_dst_g.cpu().numpy(), oracle.row_dot(Pc, a_dst, n=n_in),
          np.abs(Pc[:n_in].astype(np.float64)) @ np.abs(a_dst.astype(np.float64)), "s_dst")
    # edge softmax forward, from the GPU's own scores
    s_dst, s_src = s_dst_g.cpu().numpy(), s_src_g.cpu().numpy()
    ws = torch.empty(B.sylvie_edge_softmax_workspace_bytes(pieces[1].numel(), n_in) // 4, device=DEV)
    alpha_g = torch.full((nnz,), float("nan"), device=DEV)
    B.sylvie_edge_softmax_fwd(pieces, cld, s_dst_g, s_src_g, 0.2, alpha_g, ws)
    torch.cuda.synchronize()
    alpha = alpha_g.cpu().numpy()
    ref = oracle.edge_softmax_fwd(rp, cl, s_dst, s_src, 0.2)
    close(alpha, ref, ref, "alpha")
    # sampled product
    dZ = make_rows(rng, n_in, ld, "normal")
    dal_g = torch.full((nnz,), float("nan"), device=DEV)
    B.sylvie_sddmm(pieces, cld, dev(dZ), ld, Pd, ld, F, dal_g)
    torch.cuda.synchronize()
    dref, S = oracle.sddmm(rp, cl, np.ascontiguousarray(dZ[:, :F]), Pc, F, want_S=True)
    dalpha = dal_g.cpu().numpy()
    close(dalpha, dref, S, "dalpha")
    # softmax backward, from the GPU's alpha and dalpha
    de_g = torch.full((nnz,), float("nan"), device=DEV)
    B.sylvie_edge_softmax_bwd(pieces, cld, alpha_g, dal_g, s_dst_g, s_src_g, 0.2, de_g, ws)
    torch.cuda.synchronize()
    de_ref, Se = oracle.edge_softmax_bwd(rp, cl, alpha, dalpha, s_dst, s_src, 0.2, want_S=True)
    de = de_g.cpu().numpy()
    close(de, de_ref, Se, "de")
    # row sums on the operator, column sums through the transposed operator
    out = torch.full((n_in,), float("nan"), device=DEV)
    B.sylvie_segment_sum(pieces, de_g, out, ws)
    rs, Ss = oracle.segment_sum(rp, de, want_S=True)
    torch.cuda.synchronize()
    close(out.cpu().numpy(), rs, Ss, "ds_dst")
    *opT, perm = GE.transpose_csr(rpd, cld, torch.ones(nnz, device=DEV), n_loc, want_perm=True)
    piecesT = GE.piece_table(opT[0], chunk)
    deT = torch.empty(nnz, device=DEV)
    B.sylvie_permute_f32(de_g, perm, nnz, deT)
    outT = torch.full((n_loc,), float("nan"), device=DEV)
    wsT = torch.empty(piecesT[1].numel() + 1, device=DEV)
    B.sylvie_segment_sum(piecesT, deT, outT, wsT)
    torch.cuda.synchronize()
    cs, Sc = oracle.column_sum(rp, cl, n_loc, de, want_S=True)
    close(outT.cpu().numpy(), cs, Sc, "ds_src")
    assert np.array_equal(deT.cpu().numpy(), de[perm.cpu().numpy()])
    # rank-1 update and ReLU are exact
    X = make_rows(rng, n_loc, ld, "normal")
    Xg = dev(X)
    B.sylvie_rank1_add(Xg, ld, n_in, F, out, dev(a_dst))
    torch.cuda.synchronize()
    oracle.rank1_add(X, n_in, out.cpu().numpy(), a_dst)
    assert np.array_equal(bits32(Xg.cpu().numpy()), bits32(X))
    H = torch.full((n_in, ld), 5.0, device=DEV)
    B.sylvie_relu_fwd(dev(dZ), ld, n_in, F, H, ld)
    G = torch.full((n_in, ld), 5.0, device=DEV)
    B.sylvie_relu_bwd(H, ld, Xg, ld, n_in, F, G, ld)
    torch.cuda.synchronize()
    assert np.array_equal(H[:, :F].cpu().numpy(), np.maximum(dZ[:, :F], 0))
    assert np.array_equal(G[:, :F].cpu().numpy(), np.where(dZ[:, :F] > 0, X[:n_in, :F], 0).astype(np.float32))
    assert bool((H[:, F:] == 5.0).all()) and bool((G[:, F:] == 5.0).all())


def test_attention_kernels_degenerate(oracle):
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    # rows without entries, single-entry rows, one long row
    rp = np.array([0, 0, 1, 1, 301, 303], np.int64)
    cl = np.concatenate([[2], np.arange(300), [0, 4]]).astype(np.int32)
    rpd, cld = dev(rp), dev(cl)
    pieces = GE.piece_table(rpd, 64)
    assert pieces[1].cpu().tolist() == [1] + [3] * 5 + [4]
    rng = np.random.default_rng(0)
    s_dst = rng.standard_normal(5).astype(np.float32); s_src = rng.standard_normal(300).astype(np.float32)
    ws = torch.empty(B.sylvie_edge_softmax_workspace_bytes(pieces[1].numel(), 5) // 4, device=DEV)
    alpha = torch.zeros(303, device=DEV)
    B.sylvie_edge_softmax_fwd(pieces, cld, dev(s_dst), dev(s_src), 0.2, alpha, ws)
    out = torch.full((5,), float("nan"), device=DEV)
    B.sylvie_segment_sum(pieces, alpha, out, ws)
    torch.cuda.synchronize()
    ref = oracle.edge_softmax_fwd(rp, cl, s_dst, s_src, 0.2)
    assert np.allclose(alpha.cpu().numpy(), ref, rtol=1e-5)
    assert np.allclose(out.cpu().numpy(), [0, 1, 0, 1, 1], atol=1e-5)
    # nothing at all
    empty = GE.piece_table(dev(np.zeros(4, np.int64)), 64)
    B.sylvie_segment_sum(empty, None, out[:3], None)
    torch.cuda.synchronize()
    assert out[:3].cpu().tolist() == [0, 0, 0]


@pytest.mark.parametrize("F", [1, 7, 64, 100, 256])
@pytest.mark.parametrize("n", [0, 1, 5, 2047, 2048, 2049, 10_000])
def test_scaled_column_sum_parity(F, n):
    """out[f] = sum_i s[i] X[i][f]: the gradient of an attention vector from the projected rows
    and the summed score gradients. The plain definition in float64 is the reference."""
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(F * 13 + n)
    ld = F + (3 if F % 2 else 4)
    X = make_rows(rng, max(n, 1), ld, "heavy")
    s = rng.standard_normal(max(n, 1)).astype(np.float32)
    out = torch.full((F + 2,), 7.0, device=DEV)
    ws = torch.empty(max(B.sylvie_scaled_column_sum_workspace_bytes(n, F) // 4, 1), device=DEV)
    B.sylvie_scaled_column_sum(dev(X), ld, n, F, dev(s), out, ws)
    torch.cuda.synchronize()
    X64, s64 = X[:n, :F].astype(np.float64), s[:n].astype(np.float64)
    got = out.cpu().numpy()
    close(got[:F], (X64.T @ s64).astype(np.float32), np.abs(X64).T @ np.abs(s64), "column sum")
    assert (got[F:] == 7.0).all()


def _heads_setup(oracle, K, F, chunk, seed):
    from paper_2303_01277_amd import graph_engine as GE
    p, rp, cl, rpd, cld, pieces = setup(oracle, 20_000, chunk)
    n_in, n_loc, nnz = p.n_in, p.n_in + p.n_halo, int(rp[-1])
    rng = np.random.default_rng(seed)
    h = K * F
    ld = h + (3 if h % 2 else 4)
    P = make_rows(rng, n_loc, ld, "normal")
    dZ = make_rows(rng, n_in, ld, "normal")
    a_dst = (rng.standard_normal(h) / np.sqrt(F)).astype(np.float32)
    a_src = (rng.standard_normal(h) / np.sqrt(F)).astype(np.float32)
    *opT, perm = GE.transpose_csr(rpd, cld, torch.ones(nnz, device=DEV), n_loc, want_perm=True)
    piecesT = GE.piece_table(opT[0], chunk)
    return dict(p=p, rp=rp, cl=cl, rpd=rpd, cld=cld, pieces=pieces, piecesT=piecesT, opT=opT, perm=perm,
                n_in=n_in, n_loc=n_loc, nnz=nnz, h=h, ld=ld, P=P, dZ=dZ, a_dst=a_dst, a_src=a_src)


@pytest.mark.parametrize("chunk", [64, 1024])
@pytest.mark.parametrize("K,F", [(2, 7), (2, 64), (4, 16), (4, 64), (4, 100), (8, 32), (8, 128), (3, 7)])
def test_heads_calls_equal_single_head_calls(oracle, K, F, chunk):
    """Every K-head call against K single-head calls on the heads' own slices: bit for bit (the
    single-head calls are checked against the oracle above)."""
    from paper_2303_01277_amd import binding as B
    s = _heads_setup(oracle, K, F, chunk, 17 * K + F + chunk)
    n_in, n_loc, nnz, h, ld = s["n_in"], s["n_loc"], s["nnz"], s["h"], s["ld"]
    Pd, dZd, a_dst, a_src = dev(s["P"]), dev(s["dZ"]), dev(s["a_dst"]), dev(s["a_src"])
    pieces, piecesT, cld, perm = s["pieces"], s["piecesT"], s["cld"], s["perm"]
    new = lambda n: torch.full((n,), float("nan"), device=DEV)
    col = lambda t, k: t.view(-1, K)[:, k].contiguous()
    same = lambda a, b: torch.equal(a.view(torch.int32), b.view(torch.int32))
    # scores
    sd, ss = new(n_in * K), new(n_loc * K)
    B.sylvie_row_dot_heads(Pd, ld, n_in, F, K, a_dst, sd, a2=a_src, n2=n_loc, out2=ss)
    sd_alone = new(n_in * K)
    B.sylvie_row_dot_heads(Pd, ld, n_in, F, K, a_dst, sd_alone)
    assert same(sd, sd_alone)
    sd1, ss1 = [new(n_in) for _ in range(K)], [new(n_loc) for _ in range(K)]
    for k in range(K):
        B.sylvie_row_dot(Pd[:, k * F:], ld, n_in, F, a_dst[k * F:], sd1[k])
        B.sylvie_row_dot(Pd[:, k * F:], ld, n_loc, F, a_src[k * F:], ss1[k])
        assert same(col(sd, k), sd1[k]) and same(col(ss, k), ss1[k]), ("row_dot", k)
    # sampled product: any K; the other per-entry calls: K = 1, 2, 4, 8
    dal = new(nnz * K)
    B.sylvie_sddmm_heads(pieces, cld, dZd, ld, Pd, ld, F, K, dal)
    dal1 = [new(nnz) for _ in range(K)]
    for k in range(K):
        B.sylvie_sddmm(pieces, cld, dZd[:, k * F:], ld, Pd[:, k * F:], ld, F, dal1[k])
        assert same(col(dal, k), dal1[k]), ("sddmm", k)
    # attention-vector gradients: any K that divides the width
    sc = torch.randn(n_loc * K, device=DEV)
    ws_col = torch.empty(max(2 * B.sylvie_scaled_column_sum_workspace_bytes(n_loc, h) // 4, 1), device=DEV)
    out = torch.full((h + 2,), 7.0, device=DEV)
    B.sylvie_scaled_column_sum_heads(Pd, ld, n_loc, h, K, sc, out, ws_col)
    # two sums in one pass (the shorter one over the inner rows) keep the bits they have alone
    sc2 = torch.randn(n_in * K, device=DEV)
    o_a, o_b, o_b1 = new(h), new(h), new(h)
    B.sylvie_scaled_column_sum_heads(Pd, ld, n_in, h, K, sc2, o_b, ws_col, s2=sc, n2=n_loc, out2=o_a)
    B.sylvie_scaled_column_sum_heads(Pd, ld, n_in, h, K, sc2, o_b1, ws_col)
    assert same(o_a, out[:h].contiguous()) and same(o_b, o_b1)
    for k in range(K):
        o1 = new(F)
        B.sylvie_scaled_column_sum(Pd[:, k * F:], ld, n_loc, F, col(sc, k), o1, ws_col)
        assert same(out[k * F:(k + 1) * F], o1), ("column sum", k)
    assert bool((out[h:] == 7.0).all())
    if K == 3:
        with pytest.raises(B.SylvieError):
            B.sylvie_edge_softmax_fwd_heads(pieces, cld, sd, ss, K, 0.2, new(nnz * K), new(16))
        return
    ws = torch.empty(max(B.sylvie_edge_softmax_heads_workspace_bytes(pieces[1].numel(), n_in, K) // 4,
                         (piecesT[1].numel() + n_loc) * K), device=DEV)
    al = new(nnz * K)
    B.sylvie_edge_softmax_fwd_heads(pieces, cld, sd, ss, K, 0.2, al, ws)
    al1 = [new(nnz) for _ in range(K)]
    for k in range(K):
        B.sylvie_edge_softmax_fwd(pieces, cld, sd1[k], ss1[k], 0.2, al1[k], ws)
        assert same(col(al, k), al1[k]), ("alpha", k)
    de, dsd = new(nnz * K), new(n_in * K)
    B.sylvie_edge_softmax_bwd_heads(pieces, cld, al, dal, sd, ss, K, 0.2, de, dsd, ws)
    de_only = new(nnz * K)
    B.sylvie_edge_softmax_bwd_heads(pieces, cld, al, dal, sd, ss, K, 0.2, de_only, None, ws)
    assert same(de, de_only)
    dss = new(n_loc * K)
    B.sylvie_segment_sum_heads(piecesT, de, perm, K, dss, ws)
    dsd2 = new(n_in * K)
    B.sylvie_segment_sum_heads(pieces, de, None, K, dsd2, ws)
    assert same(dsd, dsd2)
    for k in range(K):
        de1, o1, oT, deT = new(nnz), new(n_in), new(n_loc), new(nnz)
        B.sylvie_edge_softmax_bwd(pieces, cld, al1[k], dal1[k], sd1[k], ss1[k], 0.2, de1, ws)
        assert same(col(de, k), de1), ("de", k)
        B.sylvie_segment_sum(pieces, de1, o1, ws)
        assert same(col(dsd, k), o1), ("ds_dst", k)
        B.sylvie_permute_f32(de1, perm, nnz, deT)
        B.sylvie_segment_sum(piecesT, deT, oT, ws)
        assert same(col(dss, k), oT), ("ds_src", k)
    torch.cuda.synchronize()


@pytest.mark.parametrize("chunk", [0, 64])
@pytest.mark.parametrize("K,F", [(1, 256), (2, 7), (2, 50), (4, 16), (4, 64), (4, 100), (8, 64), (3, 20), (5, 1)])
def test_attention_aggregation_parity(oracle, K, F, chunk):
    """sylvie_aggregate_csr_attention, forward (with and without the activation) and through the
    transposed operator with the entry map and the two rank-1 terms, per head against the oracle;
    the options against each other bit for bit."""
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    s = _heads_setup(oracle, K, F, 64, 31 * K + F)
    rp, cl, n_in, n_loc, nnz, h, ld = s["rp"], s["cl"], s["n_in"], s["n_loc"], s["nnz"], s["h"], s["ld"]
    rng = np.random.default_rng(K * 1000 + F)
    al = rng.random((nnz, K)).astype(np.float32)
    ald, Pd, dZd = dev(al.reshape(-1)), dev(s["P"]), dev(s["dZ"])
    rpT, clT, _ = s["opT"]
    perm = s["perm"]
    same = lambda a, b: torch.equal(a.view(torch.int32), b.view(torch.int32))

    def plan(rowptr):
        if not chunk:
            return {}
        lr, lp, nt = GE.long_row_plan(rowptr, chunk)
        assert nt > 0
        return dict(chunk=chunk, long_rows=lr, long_ptr=lp, n_long=int(lr.numel()), n_tasks=nt,
                    workspace=torch.empty(max(1, nt) * h, device=DEV))

    # forward
    kw = plan(s["rpd"])
    Z = torch.full((n_in, ld), 5.0, device=DEV)
    B.sylvie_aggregate_csr_attention(s["rpd"], s["cld"], ald, None, K, n_in, Pd, ld, h, Z, ld, **kw)
    Zr = torch.full((n_in, ld), 5.0, device=DEV)
    B.sylvie_aggregate_csr_attention(s["rpd"], s["cld"], ald, None, K, n_in, Pd, ld, h, Zr, ld, relu=True, **kw)
    torch.cuda.synchronize()
    assert same(Zr[:, :h].contiguous(), torch.where(Z[:, :h] > 0, Z[:, :h], torch.zeros_like(Z[:, :h])).contiguous())
    assert bool((Z[:, h:] == 5.0).all()) and bool((Zr[:, h:] == 5.0).all())
    Zh = Z.cpu().numpy()
    for k in range(K):
        sl = slice(k * F, (k + 1) * F)
        ref, S = oracle.aggregate_fwd(rp, cl, np.ascontiguousarray(al[:, k]), np.ascontiguousarray(s["P"][:, sl]), F,
                                      want_S=True)
        close(Zh[:, sl], ref, S, ("Z", k))
    # backward: transposed operator, weights through the entry map, rank-1 terms
    kwT = plan(rpT)
    ds_src, ds_dst = torch.randn(n_loc * K, device=DEV), torch.randn(n_in * K, device=DEV)
    a_src, a_dst = dev(s["a_src"]), dev(s["a_dst"])
    dP = torch.full((n_loc, ld), 5.0, device=DEV)
    B.sylvie_aggregate_csr_attention(rpT, clT, ald, perm, K, n_loc, dZd, ld, h, dP, ld, s1=ds_src, a1=a_src,
                                     n1=n_loc, s2=ds_dst, a2=a_dst, n2=n_in, **kwT)
    # the same without the options: weights permuted beforehand, rank-1 terms as separate calls
    alT = ald.view(nnz, K)[perm].contiguous().view(-1)
    dP2 = torch.full((n_loc, ld), 5.0, device=DEV)
    B.sylvie_aggregate_csr_attention(rpT, clT, alT, None, K, n_loc, dZd, ld, h, dP2, ld, **kwT)
    plain = dP2.clone()
    for k in range(K):
        B.sylvie_rank1_add(dP2[:, k * F:], ld, n_loc, F, ds_src.view(-1, K)[:, k].contiguous(), a_src[k * F:])
        B.sylvie_rank1_add(dP2[:, k * F:], ld, n_in, F, ds_dst.view(-1, K)[:, k].contiguous(), a_dst[k * F:])
    torch.cuda.synchronize()
    assert same(dP, dP2)
    ph = plain.cpu().numpy()
    for k in range(K):
        sl = slice(k * F, (k + 1) * F)
        ref, S = oracle.aggregate_bwd(rp, cl, np.ascontiguousarray(al[:, k]), n_loc,
                                      np.ascontiguousarray(s["dZ"][:, sl]), F, want_S=True)
        close(ph[:, sl], ref, S, ("dP", k))
    # one head, 256 columns: the plain aggregation's own order of additions
    if K == 1 and F == 256:
        Y = torch.full((n_in, ld), 5.0, device=DEV)
        B.sylvie_aggregate_csr_fwd(s["rpd"], s["cld"], ald, None, None, n_in, Pd, ld, h, Y, ld, **kw)
        torch.cuda.synchronize()
        assert same(Y, Z)


@pytest.mark.parametrize("chunk", [0, 64])
@pytest.mark.parametrize("K,F", [(1, 16), (1, 64), (1, 256), (2, 32), (2, 128), (4, 16), (4, 64), (8, 16), (8, 32)])
def test_attention_aggregation_with_sampled_product(oracle, K, F, chunk):
    """The transposed aggregation that also forms dalpha = dZ_v . P_u: the aggregate equals the
    plain call's bit for bit, the product agrees with the oracle's sampled product over the
    forward pattern per head, and every entry is written."""
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    s = _heads_setup(oracle, K, F, 64, 7 * K + F)
    rp, cl, n_in, n_loc, nnz, h, ld = s["rp"], s["cl"], s["n_in"], s["n_loc"], s["nnz"], s["h"], s["ld"]
    assert B.sylvie_aggregate_csr_attention_sddmm_supported(h, K)
    rng = np.random.default_rng(K * 100 + F)
    al = rng.random((nnz, K)).astype(np.float32)
    ald, Pd, dZd = dev(al.reshape(-1)), dev(s["P"]), dev(s["dZ"])
    rpT, clT, _ = s["opT"]
    perm = s["perm"]
    kw = {}
    if chunk:
        lr, lp, nt = GE.long_row_plan(rpT, chunk)
        assert nt > 0
        kw = dict(chunk=chunk, long_rows=lr, long_ptr=lp, n_long=int(lr.numel()), n_tasks=nt,
                  workspace=torch.empty(max(1, nt) * h, device=DEV))
    dP = torch.full((n_loc, ld), 5.0, device=DEV)
    dal = torch.full((nnz * K + 3,), float("nan"), device=DEV)
    B.sylvie_aggregate_csr_attention_sddmm(rpT, clT, ald, perm, K, n_loc, dZd, ld, h, dP, ld, Pd, ld, dal, **kw)
    dP0 = torch.full((n_loc, ld), 5.0, device=DEV)
    B.sylvie_aggregate_csr_attention(rpT, clT, ald, perm, K, n_loc, dZd, ld, h, dP0, ld, **kw)
    torch.cuda.synchronize()
    assert torch.equal(dP.view(torch.int32), dP0.view(torch.int32))
    assert bool(torch.isnan(dal[nnz * K:]).all())
    got = dal[: nnz * K].cpu().numpy().reshape(nnz, K)
    assert not np.isnan(got).any()
    for k in range(K):
        sl = slice(k * F, (k + 1) * F)
        ref, S = oracle.sddmm(rp, cl, np.ascontiguousarray(s["dZ"][:, sl]), np.ascontiguousarray(s["P"][:, sl]), F,
                              want_S=True)
        close(got[:, k], ref, S, ("dalpha", k))
    # shapes without such a launch are refused, not mis-computed
    assert not B.sylvie_aggregate_csr_attention_sddmm_supported(24, 3)
    assert not B.sylvie_aggregate_csr_attention_sddmm_supported(512, 2)
    with pytest.raises(B.SylvieError):
        B.sylvie_aggregate_csr_attention_sddmm(rpT, clT, ald, perm, 1, n_loc, dZd, ld, 24, dP, ld, Pd, ld, dal)


def test_rank1_add_heads_equals_single_calls():
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(3)
    for K, F, n1, n2 in ((4, 64, 1000, 700), (2, 7, 333, 333), (1, 5, 10, 0), (8, 4, 64, 100)):
        h = K * F
        ld = h + (3 if h % 2 else 4)
        n = max(n1, n2)
        X = dev(make_rows(rng, n + 2, ld, "normal"))
        s1, s2 = torch.randn(n1 * K, device=DEV), torch.randn(max(n2, 1) * K, device=DEV)
        a1, a2 = torch.randn(h, device=DEV), torch.randn(h, device=DEV)
        want = X.clone()
        for k in range(K):
            B.sylvie_rank1_add(want[:, k * F:], ld, n1, F, s1.view(-1, K)[:, k].contiguous(), a1[k * F:])
            if n2:
                B.sylvie_rank1_add(want[:, k * F:], ld, n2, F, s2.view(-1, K)[:, k].contiguous(), a2[k * F:])
        B.sylvie_rank1_add_heads(X, ld, h, K, s1, a1, n1, s2 if n2 else None, a2 if n2 else None, n2)
        torch.cuda.synchronize()
        assert torch.equal(X.view(torch.int32), want.view(torch.int32)), (K, F)


def test_attention_aggregation_rejects_bad_arguments():
    from paper_2303_01277_amd import binding as B
    rp = dev(np.array([0, 1, 2], np.int64)); cl = dev(np.array([0, 1], np.int32))
    w = torch.ones(2 * 9, device=DEV); X = torch.ones(2, 72, device=DEV); Y = torch.empty(2, 72, device=DEV)
    with pytest.raises(B.SylvieError):      # more heads than the weight table holds
        B.sylvie_aggregate_csr_attention(rp, cl, w, None, 9, 2, X, 72, 72, Y, 72)
    with pytest.raises(B.SylvieError):      # heads must divide d
        B.sylvie_aggregate_csr_attention(rp, cl, w, None, 5, 2, X, 72, 72, Y, 72)
    with pytest.raises(B.SylvieError):      # a rank-1 term without its vector
        B.sylvie_aggregate_csr_attention(rp, cl, w, None, 2, 2, X, 72, 72, Y, 72, s1=w)
    B.sylvie_aggregate_csr_attention(rp, cl, w, None, 2, 2, X, 72, 72, Y, 72)
    torch.cuda.synchronize()
    assert bool((Y == 1.0).all())
