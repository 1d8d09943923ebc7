"""Pins for the oracle's normalised operators, aggregation and its transpose
(Eq. 1; Sec. 3.4, A_hat = D^-1/2 (A + I) D^-1/2; Alg. 2 feature gradients)."""
import numpy as np
import scipy.sparse as sp
import torch

from synth import CONFIGS, build_workload, scaled, er_edges, partition_by_range
from util import np_c, to_partdata


def dense_adj(n, u, v):
    A = np.zeros((n, n))
    A[u, v] = 1.0
    A[v, u] = 1.0
    return A


def small_graph(n=60, deg=6.0, seed=3, parts=3):
    u, v = er_edges(n, deg, seed)
    P = [partition_by_range(u, v, n, parts, p) for p in range(parts)]
    return np_c(u), np_c(v), P


def test_gcn_operator_vs_dense_bruteforce(oracle):
    n = 60
    u, v, P = small_graph(n)
    A = dense_adj(n, u, v) + np.eye(n)
    dinv = 1.0 / np.sqrt(A.sum(1))
    Ahat = dinv[:, None] * A * dinv[None, :]
    assert np.allclose(Ahat, Ahat.T)
    for p in P:
        rp, cl, w = oracle.gcn_operator(np_c(p.rowptr), np_c(p.col), np_c(p.deg), p.n_in)
        assert rp[-1] == p.nnz + p.n_in
        gid = np.concatenate([np.arange(p.lo, p.lo + p.n_in), np_c(p.halo_gid)])
        got = np.zeros((p.n_in, n))
        for r in range(p.n_in):
            cols = cl[rp[r]:rp[r + 1]]
            assert (np.diff(cols) > 0).all()                    # sorted, self loop in place
            assert r in cols
            got[r, gid[cols]] = w[rp[r]:rp[r + 1]]
        assert np.abs(got - Ahat[p.lo:p.lo + p.n_in]).max() < 1e-7
        # weights are the double-precision value rounded once
        for r in range(p.n_in):
            for e in range(rp[r], rp[r + 1]):
                assert w[e] == np.float32(Ahat[p.lo + r, gid[cl[e]]])


def test_gcn_regular_graph_ones(oracle):
    # ring of 40 nodes (2-regular): A_hat * 1 = 1
    n = 40
    u = torch.arange(n)
    v = (u + 1) % n
    lo, hi = torch.minimum(u, v), torch.maximum(u, v)
    for parts in (1, 4):
        for pi in range(parts):
            p = partition_by_range(lo, hi, n, parts, pi)
            rp, cl, w = oracle.gcn_operator(np_c(p.rowptr), np_c(p.col), np_c(p.deg), p.n_in)
            X = np.ones((p.n_in + p.n_halo, 5), np.float32)
            Z = oracle.aggregate_fwd(rp, cl, w, X, 5)
            assert np.abs(Z - 1.0).max() < 1e-6


def test_mean_of_ones_is_ones(oracle):
    u, v, P = small_graph(80, 5.0, 5, 2)
    for p in P:
        rp, cl = np_c(p.rowptr), np_c(p.col)
        w = oracle.mean_weights(rp, p.n_in)
        X = np.ones((p.n_in + p.n_halo, 3), np.float32)
        Z = oracle.aggregate_fwd(rp, cl, w, X, 3)
        has = np.diff(rp) > 0
        assert np.abs(Z[has] - 1.0).max() < 1e-6
        assert (Z[~has] == 0).all()


def test_aggregate_vs_scipy_and_adjoint(oracle):
    wl = build_workload(scaled(CONFIGS["citation"], 3000))
    p = to_partdata(wl)[0]
    rp, cl, w = oracle.gcn_operator(p.rowptr, p.col, p.deg, p.n_in)
    ncols = p.n_in + p.n_halo
    A = sp.csr_matrix((w.astype(np.float64), cl, rp), shape=(p.n_in, ncols))
    rng = np.random.default_rng(0)
    d = 37
    X = rng.standard_normal((ncols, d)).astype(np.float32)
    Z, S = oracle.aggregate_fwd(rp, cl, w, X, d, want_S=True)
    ref = A @ X.astype(np.float64)
    assert np.array_equal(Z, ref.astype(np.float32)) or np.abs(Z - ref).max() <= 1e-7 * np.abs(
        ref).max()
    assert np.allclose(S, abs(A) @ np.abs(X.astype(np.float64)), rtol=1e-6)
    dZ = rng.standard_normal((p.n_in, d)).astype(np.float32)
    dX, Sb = oracle.aggregate_bwd(rp, cl, w, ncols, dZ, d, want_S=True)
    refb = A.T @ dZ.astype(np.float64)
    assert np.abs(dX - refb).max() <= 1e-7 * np.abs(refb).max()
    # adjoint identity <A x, y> = <x, A^T y>
    lhs = (Z.astype(np.float64) * dZ).sum()
    rhs = (X.astype(np.float64) * dX).sum()
    assert abs(lhs - rhs) <= 1e-6 * max(abs(lhs), (S.astype(np.float64) * np.abs(dZ)).sum())
    # the sampled-row variant agrees with the full one
    sel = np.unique(rng.integers(0, ncols, 50)).astype(np.int32)
    out, So = oracle.aggregate_bwd_rows(rp, cl, w, dZ, d, sel)
    assert np.array_equal(out, dX[sel]) and np.array_equal(So, Sb[sel])


def test_leading_dimension(oracle):
    u, v, P = small_graph(50, 4.0, 8, 2)
    p = P[0]
    rp, cl = np_c(p.rowptr), np_c(p.col)
    w = oracle.mean_weights(rp, p.n_in)
    rng = np.random.default_rng(1)
    X = rng.standard_normal((p.n_in + p.n_halo, 20)).astype(np.float32)
    Z_all = oracle.aggregate_fwd(rp, cl, w, X, 20)
    Z_12 = oracle.aggregate_fwd(rp, cl, w, X, 12)               # reads ld = 20, d = 12
    assert np.array_equal(Z_12, Z_all[:, :12])
