"""Pins for the oracle's Graph Engine set-up (Alg. 1, the lines before the epoch loop: HALO set,
send / receive sets; Sec. 3.2): numpy's set routines, scipy's sparse transpose, a stable argsort,
and the identities that tie the sets of different partitions together."""
import numpy as np
import pytest
import scipy.sparse as sp


def random_partitioned_graph(rng, n_nodes, n_parts, avg_deg, contiguous):
    m = int(n_nodes * avg_deg / 2)
    u = rng.integers(0, n_nodes, m); v = rng.integers(0, n_nodes, m)
    keep = u != v
    A = sp.coo_matrix((np.ones(keep.sum() * 2), (np.r_[u[keep], v[keep]], np.r_[v[keep], u[keep]])),
                      shape=(n_nodes, n_nodes)).tocsr()
    A.sum_duplicates(); A.sort_indices()
    if contiguous:
        owner = (np.arange(n_nodes) * n_parts // n_nodes).astype(np.int32)
    else:
        owner = rng.integers(0, n_parts, n_nodes).astype(np.int32)
    return A, owner


def subgraph(A, owner, part):
    mine = np.flatnonzero(owner == part)
    sub = A[mine]
    return mine, sub.indptr.astype(np.int64), sub.indices.astype(np.int32)


@pytest.mark.parametrize("contiguous", [True, False])
@pytest.mark.parametrize("n_parts", [1, 2, 5])
def test_halo_and_exchange_sets_against_set_routines(oracle, contiguous, n_parts):
    rng = np.random.default_rng(n_parts + 10 * contiguous)
    A, owner = random_partitioned_graph(rng, 400, n_parts, 5.0, contiguous)
    row_of, part_ptr = oracle.rows_in_owner(owner, n_parts)
    assert np.array_equal(part_ptr, np.r_[0, np.cumsum(np.bincount(owner, minlength=n_parts))])
    halos, poss = [], []
    for n in range(n_parts):
        mine, rp, gc = subgraph(A, owner, n)
        assert np.array_equal(row_of[mine], np.arange(mine.size))
        halo, pos, n_inner = oracle.halo_set(rp, gc, mine.size, owner, n)
        # line 3: { v in G_n : v not in V_n }
        assert np.array_equal(halo, np.setdiff1d(np.unique(gc), mine))
        assert n_inner == mine.size
        assert np.array_equal(pos[mine], np.arange(mine.size))
        assert np.array_equal(pos[halo], mine.size + np.arange(halo.size))
        rest = np.setdiff1d(np.arange(400), np.r_[mine, halo])
        assert (pos[rest] == -1).all()
        col = oracle.relabel_columns(gc, pos)
        local_gid = np.r_[mine, halo]
        assert np.array_equal(local_gid[col], gc) and col.min(initial=0) >= 0
        halos.append(halo); poss.append(pos)
    for n in range(n_parts):
        mine = np.flatnonzero(owner == n)
        R_ptr, R_halo, R_row = oracle.recv_sets(halos[n], owner, row_of, n_parts)
        assert R_ptr[0] == 0 and R_ptr[-1] == halos[n].size and R_ptr[n] == R_ptr[n + 1]
        for k in range(n_parts):
            theirs = np.flatnonzero(owner == k)
            Rk = halos[n][R_halo[R_ptr[k]:R_ptr[k + 1]]]
            assert np.array_equal(Rk, np.intersect1d(halos[n], theirs))           # line 7
            assert np.array_equal(theirs[R_row[R_ptr[k]:R_ptr[k + 1]]], Rk)
            Sk = oracle.send_set(halos[k], owner, row_of, n)
            assert np.array_equal(mine[Sk], np.intersect1d(mine, halos[k]))        # line 6
        # what n receives from k is what k sends to n, row for row
        for k in range(n_parts):
            Rk_ptr, _, Rk_row = oracle.recv_sets(halos[k], owner, row_of, n_parts)
            assert np.array_equal(oracle.send_set(halos[k], owner, row_of, n), Rk_row[Rk_ptr[n]:Rk_ptr[n + 1]])


def test_halo_set_matches_the_input_generator(oracle):
    """The synthetic partitions were cut by a different route (torch, id ranges): same halo set,
    same numbering of the halo rows, same owner and row of every halo node."""
    from synth import CONFIGS, build_workload, scaled
    import dataclasses
    spec = dataclasses.replace(scaled(CONFIGS["tiny"], 600, 6.0), all_parts=True, n_parts=3)
    wl = build_workload(spec)
    n_nodes = 600
    width = -(-n_nodes // 3)
    owner = (np.arange(n_nodes) // width).astype(np.int32)
    row_of, _ = oracle.rows_in_owner(owner, 3)
    for p in wl.parts:
        rp = p.rowptr.numpy().astype(np.int64)
        local_gid = np.r_[p.lo + np.arange(p.n_in), p.halo_gid.numpy()]
        gcol = local_gid[p.col.numpy()].astype(np.int32)
        halo, pos, n_inner = oracle.halo_set(rp, gcol, p.n_in, owner, p.part)
        assert n_inner == p.n_in and np.array_equal(halo, p.halo_gid.numpy())
        assert np.array_equal(oracle.relabel_columns(gcol, pos), p.col.numpy())
        R_ptr, R_halo, R_row = oracle.recv_sets(halo, owner, row_of, 3)
        got_owner = np.empty(halo.size, np.int32); got_row = np.empty(halo.size, np.int32)
        for k in range(3):
            got_owner[R_halo[R_ptr[k]:R_ptr[k + 1]]] = k
            got_row[R_halo[R_ptr[k]:R_ptr[k + 1]]] = R_row[R_ptr[k]:R_ptr[k + 1]]
        assert np.array_equal(got_owner, p.halo_part.numpy()) and np.array_equal(got_row, p.halo_row.numpy())


@pytest.mark.parametrize("shape", [(1, 1), (7, 3), (50, 80), (300, 40), (64, 64)])
def test_transpose_against_scipy(oracle, shape):
    rng = np.random.default_rng(shape[0])
    n_rows, n_cols = shape
    A = sp.random(n_rows, n_cols, density=0.2, random_state=np.random.RandomState(shape[1]), format="csr",
                  data_rvs=lambda k: rng.standard_normal(k).astype(np.float32)).astype(np.float32)
    A.sort_indices()
    rp, cl, w = A.indptr.astype(np.int64), A.indices.astype(np.int32), A.data.astype(np.float32)
    rpT, clT, wT, perm = oracle.transpose_csr(rp, cl, w, n_cols)
    T = A.T.tocsr(); T.sort_indices()
    assert np.array_equal(rpT, T.indptr) and np.array_equal(clT, T.indices) and np.array_equal(wT, T.data)
    assert np.array_equal(w[perm], wT) and np.array_equal(np.sort(perm), np.arange(cl.size))
    # a stable sort of the entries by column is the same statement
    assert np.array_equal(perm, np.argsort(cl, kind="stable"))
    # transposing twice gives the operator back; no weights is allowed
    rp2, cl2, w2, _ = oracle.transpose_csr(rpT, clT, wT, n_rows)
    assert np.array_equal(rp2, rp) and np.array_equal(cl2, cl) and np.array_equal(w2, w)
    assert oracle.transpose_csr(rp, cl, None, n_cols)[2] is None


def test_transpose_unsorted_rows_and_empty(oracle):
    """Columns of a row need not ascend (the halo columns of a relabelled row do not); duplicates
    keep their order; an operator without entries gives an all-zero row pointer."""
    rp = np.array([0, 3, 3, 6], np.int64)
    cl = np.array([2, 0, 2, 1, 2, 0], np.int32)
    w = np.arange(6, dtype=np.float32)
    rpT, clT, wT, perm = oracle.transpose_csr(rp, cl, w, 4)
    assert rpT.tolist() == [0, 2, 3, 6, 6]
    assert clT.tolist() == [0, 2, 2, 0, 0, 2] and perm.tolist() == [1, 5, 3, 0, 2, 4]
    assert wT.tolist() == [1, 5, 3, 0, 2, 4]
    rpT, clT, _, perm = oracle.transpose_csr(np.zeros(4, np.int64), np.zeros(0, np.int32), None, 5)
    assert rpT.tolist() == [0] * 6 and clT.size == 0 and perm.size == 0


def test_scatter_segments_against_stable_sort(oracle):
    rng = np.random.default_rng(5)
    dst = rng.integers(0, 37, 500).astype(np.int32)
    dst[:60] = 11
    seg_ptr, seg_rows = oracle.scatter_segments(dst, 40)
    assert np.array_equal(seg_rows, np.argsort(dst, kind="stable"))
    assert np.array_equal(seg_ptr, np.r_[0, np.cumsum(np.bincount(dst, minlength=40))])
    sp_, sr = oracle.scatter_segments(np.zeros(0, np.int32), 3)
    assert sp_.tolist() == [0, 0, 0, 0] and sr.size == 0
