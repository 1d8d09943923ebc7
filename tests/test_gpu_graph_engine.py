"""GPU parity of the device Graph Engine (HALO set, local numbering, receive sets, transposed
operator, scatter segments) against the CPU oracle: integer results, compared exactly, on sizes
that span several sort tiles, several digits and a ragged tail."""
import numpy as np
import pytest
import torch

from test_gpu_ops import DEV, dev

pytestmark = pytest.mark.gpu


def workspace(B, n):
    return torch.empty(B.sylvie_graph_workspace_bytes(n) // 8 + 1, dtype=torch.int64, device=DEV)


def random_csr(rng, n_rows, n_cols, avg, hub=0):
    counts = rng.poisson(avg, n_rows).astype(np.int64)
    if n_rows >= 10:
        counts[rng.integers(0, n_rows, n_rows // 10)] = 0               # empty rows
    counts[0] = max(counts[0], 1)
    if hub:
        counts[n_rows // 3] = hub
    rp = np.r_[0, np.cumsum(counts)].astype(np.int64)
    zipf = (n_cols * rng.random(int(rp[-1])) ** 3).astype(np.int64)     # skewed columns
    return rp, np.minimum(zipf, n_cols - 1).astype(np.int32)


@pytest.mark.parametrize("n_rows,n_cols,avg,hub", [
    (1, 1, 3, 0), (5, 3, 2, 0), (300, 257, 4, 0), (2000, 70_000, 9, 5000), (40_000, 300, 6, 0),
    (30_000, 1 << 17, 16, 20_000)])
def test_transpose_csr_parity(oracle, n_rows, n_cols, avg, hub):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(n_rows + n_cols)
    rp, cl = random_csr(rng, n_rows, n_cols, avg, hub)
    nnz = int(rp[-1])
    w = rng.standard_normal(nnz).astype(np.float32)
    ref = oracle.transpose_csr(rp, cl, w, n_cols)
    rpT = torch.full((n_cols + 2,), -7, dtype=torch.int64, device=DEV)
    clT = torch.full((nnz + 1,), -7, dtype=torch.int32, device=DEV)
    wT = torch.full((nnz + 1,), -7.0, device=DEV)
    perm = torch.full((nnz + 1,), -7, dtype=torch.int64, device=DEV)
    ws = workspace(B, nnz)
    B.sylvie_graph_transpose_csr(dev(rp), dev(cl), dev(w), n_rows, n_cols, nnz, rpT, clT, wT, perm, ws)
    assert np.array_equal(rpT.cpu().numpy()[:-1], ref[0]) and int(rpT[-1]) == -7
    assert np.array_equal(clT.cpu().numpy()[:-1], ref[1]) and int(clT[-1]) == -7
    assert np.array_equal(wT.cpu().numpy()[:-1], ref[2]) and float(wT[-1]) == -7.0
    assert np.array_equal(perm.cpu().numpy()[:-1], ref[3]) and int(perm[-1]) == -7
    # without weights and without the permutation; twice gives the operator back when the
    # columns of every row ascend
    clT2 = torch.empty(nnz + 1, dtype=torch.int32, device=DEV)
    rpT2 = torch.empty(n_cols + 1, dtype=torch.int64, device=DEV)
    B.sylvie_graph_transpose_csr(dev(rp), dev(cl), None, n_rows, n_cols, nnz, rpT2, clT2, None, None, ws)
    assert torch.equal(rpT2, rpT[:-1]) and torch.equal(clT2[:nnz], clT[:nnz])


def test_transpose_rejects_bad_input(oracle):
    from paper_2303_01277_amd import binding as B
    rp = np.array([0, 2, 4], np.int64); cl = np.array([0, 1, 5, 1], np.int32)
    out = [torch.empty(4, dtype=torch.int64, device=DEV), torch.empty(4, dtype=torch.int32, device=DEV)]
    ws = workspace(B, 4)
    with pytest.raises(B.SylvieError, match="column outside"):
        B.sylvie_graph_transpose_csr(dev(rp), dev(cl), None, 2, 3, 4, out[0], out[1], None, None, ws)
    cl[2] = 2
    with pytest.raises(B.SylvieError, match="row pointer"):
        B.sylvie_graph_transpose_csr(dev(rp), dev(cl), None, 2, 3, 3, out[0], out[1], None, None, ws)
    with pytest.raises(B.SylvieError, match="workspace"):
        B.sylvie_graph_transpose_csr(dev(rp), dev(cl), None, 2, 3, 4, out[0], out[1], None, None, ws[:8])
    # an operator without entries
    rp0 = np.zeros(4, np.int64)
    rpT = torch.full((6,), -1, dtype=torch.int64, device=DEV)
    B.sylvie_graph_transpose_csr(dev(rp0), None, None, 3, 5, 0, rpT, None, None, None, ws)
    assert rpT.tolist() == [0] * 6


@pytest.mark.parametrize("n,n_dst", [(0, 4), (1, 1), (517, 40), (5000, 3000), (70_000, 300), (70_000, 1 << 18)])
def test_scatter_segments_parity(oracle, n, n_dst):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(n + n_dst)
    dst = rng.integers(0, n_dst, n).astype(np.int32)
    dst[: n // 10] = n_dst // 2
    ref = oracle.scatter_segments(dst, n_dst)
    seg_ptr = torch.empty(n_dst + 1, dtype=torch.int64, device=DEV)
    seg_rows = torch.full((n + 1,), -3, dtype=torch.int32, device=DEV)
    B.sylvie_graph_scatter_segments(dev(dst) if n else None, n, n_dst, seg_ptr, seg_rows, workspace(B, n))
    assert np.array_equal(seg_ptr.cpu().numpy(), ref[0])
    assert np.array_equal(seg_rows.cpu().numpy()[:n], ref[1]) and int(seg_rows[n]) == -3


@pytest.mark.parametrize("contiguous", [True, False])
@pytest.mark.parametrize("n_nodes,n_parts,avg", [(50, 1, 3.0), (3000, 3, 6.0), (40_000, 8, 12.0), (25_000, 300, 5.0)])
def test_halo_and_receive_sets_parity(oracle, n_nodes, n_parts, avg, contiguous):
    from paper_2303_01277_amd import binding as B
    rng = np.random.default_rng(n_nodes + n_parts + contiguous)
    if contiguous:
        owner = (np.arange(n_nodes) * n_parts // n_nodes).astype(np.int32)
    else:
        owner = rng.integers(0, n_parts, n_nodes).astype(np.int32)
    ow = dev(owner)
    ws = workspace(B, max(n_nodes, int(n_nodes * avg * 2)))
    row_of = torch.empty(n_nodes, dtype=torch.int32, device=DEV)
    part_ptr = torch.empty(n_parts + 1, dtype=torch.int64, device=DEV)
    B.sylvie_graph_rows_in_owner(ow, n_nodes, n_parts, row_of, part_ptr, ws)
    ref_row_of, ref_ptr = oracle.rows_in_owner(owner, n_parts)
    assert np.array_equal(row_of.cpu().numpy(), ref_row_of) and np.array_equal(part_ptr.cpu().numpy(), ref_ptr)
    for part in sorted({0, n_parts // 2, n_parts - 1}):
        mine = np.flatnonzero(owner == part)
        n_in = mine.size
        nnz = int(n_in * avg)
        gcol = rng.integers(0, n_nodes, nnz).astype(np.int32)              # neighbours, any order, repeats
        rp = np.r_[0, np.sort(rng.integers(0, nnz + 1, max(n_in - 1, 0))), nnz].astype(np.int64)[: n_in + 1]
        halo, pos_ref, n_inner = oracle.halo_set(rp, gcol, n_in, owner, part)
        pos = torch.full((n_nodes + 1,), -9, dtype=torch.int32, device=DEV)
        halo_gid = torch.full((halo.size + 1,), -9, dtype=torch.int32, device=DEV)
        counts = B.sylvie_graph_local_index(dev(gcol) if nnz else None, nnz, n_in, ow, n_nodes, part, pos,
                                            halo_gid, halo.size, ws)
        assert counts == (n_in, halo.size)
        assert np.array_equal(pos.cpu().numpy()[:-1], pos_ref) and int(pos[-1]) == -9
        assert np.array_equal(halo_gid.cpu().numpy()[:-1], halo) and int(halo_gid[-1]) == -9
        if nnz:
            col = torch.empty(nnz, dtype=torch.int32, device=DEV)
            B.sylvie_graph_relabel_columns(dev(gcol), nnz, pos, n_nodes, col, ws)
            assert np.array_equal(col.cpu().numpy(), oracle.relabel_columns(gcol, pos_ref))
        R_ptr = torch.empty(n_parts + 1, dtype=torch.int64, device=DEV)
        R_halo = torch.full((halo.size + 1,), -9, dtype=torch.int32, device=DEV)
        R_row = torch.full((halo.size + 1,), -9, dtype=torch.int32, device=DEV)
        B.sylvie_graph_recv_sets(halo_gid[:-1], halo.size, ow, row_of, n_nodes, n_parts, R_ptr, R_halo, R_row, ws)
        ref = oracle.recv_sets(halo, owner, ref_row_of, n_parts)
        assert np.array_equal(R_ptr.cpu().numpy(), ref[0])
        assert np.array_equal(R_halo.cpu().numpy()[:-1], ref[1]) and np.array_equal(R_row.cpu().numpy()[:-1], ref[2])
        # the send set toward a peer is the peer's receive slice for this partition
        peer = (part + 1) % n_parts
        if peer != part:
            sl = slice(int(ref[0][peer]), int(ref[0][peer + 1]))
            assert np.array_equal(R_row.cpu().numpy()[sl], oracle.send_set(halo, owner, ref_row_of, peer))


def test_local_index_rejects_bad_input(oracle):
    from paper_2303_01277_amd import binding as B
    owner = dev(np.array([0, 0, 1, 1, 1], np.int32))
    pos = torch.empty(5, dtype=torch.int32, device=DEV)
    halo = torch.empty(5, dtype=torch.int32, device=DEV)
    ws = workspace(B, 16)
    with pytest.raises(B.SylvieError, match="neighbour id"):
        B.sylvie_graph_local_index(dev(np.array([1, 7], np.int32)), 2, 2, owner, 5, 0, pos, halo, 5, ws)
    with pytest.raises(B.SylvieError, match="owns 2 nodes"):
        B.sylvie_graph_local_index(dev(np.array([1, 3], np.int32)), 2, 3, owner, 5, 0, pos, halo, 5, ws)
    with pytest.raises(B.SylvieError, match="room for 1"):
        B.sylvie_graph_local_index(dev(np.array([2, 3], np.int32)), 2, 2, owner, 5, 0, pos, halo, 1, ws)
    assert B.sylvie_graph_local_index(dev(np.array([2, 3, 2], np.int32)), 3, 2, owner, 5, 0, pos, halo, 2, ws) == (2, 2)
    assert pos.tolist() == [0, 1, 2, 3, -1] and halo[:2].tolist() == [2, 3]
    col = torch.empty(2, dtype=torch.int32, device=DEV)
    with pytest.raises(B.SylvieError, match="neither an inner nor a halo"):
        B.sylvie_graph_relabel_columns(dev(np.array([2, 4], np.int32)), 2, pos, 5, col, ws)
    row_of = torch.empty(5, dtype=torch.int32, device=DEV)
    pp = torch.empty(2, dtype=torch.int64, device=DEV)
    with pytest.raises(B.SylvieError, match="owner outside"):
        B.sylvie_graph_rows_in_owner(owner, 5, 1, row_of, pp, ws)
    seg = torch.empty(3, dtype=torch.int64, device=DEV)
    rows = torch.empty(2, dtype=torch.int32, device=DEV)
    with pytest.raises(B.SylvieError, match="destination row"):
        B.sylvie_graph_scatter_segments(dev(np.array([0, 2], np.int32)), 2, 2, seg, rows, ws)


def test_partitions_rebuilt_by_the_library_match_the_input_generator(oracle):
    """The synthetic partitions were cut by torch code in the input generator; the library's
    set-up, given only each partition's adjacency in global ids and the ownership array,
    arrives at the same halo sets, columns, owners and rows — and its transposes and segments
    are the ones the layer loop then uses."""
    import dataclasses
    from synth import CONFIGS, build_workload, scaled
    from paper_2303_01277_amd import graph_engine as GE
    n_nodes, n_parts = 9000, 3
    spec = dataclasses.replace(scaled(CONFIGS["tiny"], n_nodes, 8.0), all_parts=True, n_parts=n_parts)
    wl = build_workload(spec, device=DEV)
    width = -(-n_nodes // n_parts)
    owner = (torch.arange(n_nodes, device=DEV) // width).to(torch.int32)
    row_of, part_ptr = GE.rows_in_owner(owner, n_parts)
    assert part_ptr.tolist() == [0] + [min(n_nodes, (k + 1) * width) for k in range(n_parts)]
    results = []
    for p in wl.parts:
        local_gid = torch.cat([p.lo + torch.arange(p.n_in, device=DEV), p.halo_gid])
        gcol = local_gid[p.col.long()].to(torch.int32)
        pos, halo_gid, col = GE.local_index(gcol, p.n_in, owner, p.part)
        assert torch.equal(halo_gid.long(), p.halo_gid) and torch.equal(col, p.col)
        R_ptr, R_halo, R_row = GE.recv_sets(halo_gid, owner, row_of, n_parts)
        got_owner = torch.repeat_interleave(torch.arange(n_parts, device=DEV), R_ptr[1:] - R_ptr[:-1])
        assert torch.equal(R_halo.long(), torch.arange(p.n_halo, device=DEV))      # id ranges: already grouped
        assert torch.equal(got_owner.to(torch.int32), p.halo_part) and torch.equal(R_row, p.halo_row)
        results.append((R_ptr, R_row))
        # transpose against the oracle on the real operator
        rp, cl, w = GE.gcn_operator(p.rowptr, p.col, p.deg, p.n_in)
        n_loc = p.n_in + p.n_halo
        rpT, clT, wT, perm = GE.transpose_csr(rp, cl, w, n_loc, want_perm=True)
        ref = oracle.transpose_csr(rp.cpu().numpy(), cl.cpu().numpy(), w.cpu().numpy(), n_loc)
        for got, want in zip((rpT, clT, wT, perm), ref):
            assert np.array_equal(got.cpu().numpy(), want)
    # send sets: what n sends to k is k's receive slice for n (Alg. 1: S_k = V_n & V_HALO,k)
    for n in range(n_parts):
        for k in range(n_parts):
            R_ptr, R_row = results[k]
            S = R_row[int(R_ptr[n]):int(R_ptr[n + 1])].cpu().numpy()
            want = oracle.send_set(wl.parts[k].halo_gid.to(torch.int32).cpu().numpy(), owner.cpu().numpy(),
                                   row_of.cpu().numpy(), n)
            assert np.array_equal(S, want)


@pytest.mark.parametrize("cfg,n_nodes", [("citation", 4000), ("stress", 30_000), ("co_purchase", 12_000)])
def test_operator_weights_and_launch_plans(oracle, cfg, n_nodes):
    """The normalised operator (Sec. 3.4) and the mean weights against the oracle bit for bit, and
    the launch plans (long rows, pieces, longest-first order) against plain counts."""
    from synth import CONFIGS, build_workload, scaled
    from paper_2303_01277_amd import graph_engine as GE
    wl = build_workload(scaled(CONFIGS[cfg], n_nodes))
    p = wl.parts[0]
    rpd, cld, dgd = p.rowptr.to(DEV), p.col.to(DEV), p.deg.to(DEV)
    rp, cl, w = GE.gcn_operator(rpd, cld, dgd, p.n_in)
    orp, ocl, ow = oracle.gcn_operator(p.rowptr.numpy(), p.col.numpy(), p.deg.numpy(), p.n_in)
    assert np.array_equal(rp.cpu().numpy(), orp) and np.array_equal(cl.cpu().numpy(), ocl)
    assert np.array_equal(w.cpu().numpy().view(np.uint32), ow.view(np.uint32))
    _, _, wm = GE.mean_operator(rpd, cld, p.n_in)
    assert np.array_equal(wm.cpu().numpy().view(np.uint32),
                          oracle.mean_weights(p.rowptr.numpy(), p.n_in).view(np.uint32))
    cnt = np.diff(orp)
    for chunk in (64, 1024):
        lr, lp, nt = GE.long_row_plan(rp, chunk)
        assert np.array_equal(lr.cpu().numpy(), np.nonzero(cnt > chunk)[0])
        tasks = -(-cnt[cnt > chunk] // chunk)
        assert nt == int(tasks.sum()) and np.array_equal(lp.cpu().numpy(), np.concatenate([[0], np.cumsum(tasks)]))
    lo, hi = p.n_in // 3, p.n_in - 5
    lr, lp, nt = GE.long_row_plan(rp, 64, lo, hi, nnz=int(orp[hi] - orp[lo]))
    sel = np.nonzero(cnt[lo:hi] > 64)[0] + lo
    assert np.array_equal(lr.cpu().numpy(), sel) and nt == int((-(-cnt[sel] // 64)).sum())
    for chunk in (16, 1000):
        pp, pr, rpc = GE.piece_table(rp, chunk)
        per = -(-cnt // chunk)
        assert np.array_equal(np.diff(rpc.cpu().numpy()), per) and int(rpc[0]) == 0
        assert np.array_equal(pr.cpu().numpy(), np.repeat(np.arange(cnt.size), per))
        starts = np.concatenate([orp[r] + chunk * np.arange(per[r]) for r in range(cnt.size)] + [[orp[-1]]])
        assert np.array_equal(pp.cpu().numpy(), starts)
    for r0, r1 in ((0, p.n_in), (lo, hi)):
        order = GE.rows_by_length(rp, r0, r1).cpu().numpy()
        assert np.array_equal(order, np.argsort(-cnt[r0:r1], kind="stable"))


def test_operator_rejects_bad_adjacency():
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    rp = torch.tensor([0, 2, 3], dtype=torch.int64, device=DEV)
    deg = torch.tensor([2, 1, 1], dtype=torch.int32, device=DEV)
    with pytest.raises(B.SylvieError, match="self loop"):
        GE.gcn_operator(rp, torch.tensor([0, 2, 2], dtype=torch.int32, device=DEV), deg, 2)
    with pytest.raises(B.SylvieError, match="self loop"):
        GE.gcn_operator(rp, torch.tensor([1, 7, 2], dtype=torch.int32, device=DEV), deg, 2)
    with pytest.raises(B.SylvieError, match="ascend"):
        GE.gcn_operator(torch.tensor([0, 3, 2], dtype=torch.int64, device=DEV),
                        torch.tensor([1, 2, 2], dtype=torch.int32, device=DEV), deg, 2)
