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
