"""Pins for the oracle's attention aggregator (the GAT model the paper evaluates, Sec. 2.1 /
Sec. 4): library softmax and autograd on dense masked matrices, dense matmuls, and central
finite differences through the whole two-partition layer loop."""
import numpy as np
import pytest
import scipy.sparse as sp
import torch
from scipy.special import softmax

from oracle import layers as OL
from synth import CONFIGS, build_workload, scaled
from util import np_c, to_partdata


def random_pattern(rng, n_rows, n_cols, p=0.3):
    A = sp.random(n_rows, n_cols, density=p, random_state=np.random.RandomState(int(rng.integers(1 << 30))), format="csr")
    A = A + sp.eye(n_rows, n_cols, format="csr")                    # every row has an entry
    A.sort_indices()
    return A.indptr.astype(np.int64), A.indices.astype(np.int32)


def test_edge_softmax_against_library(oracle):
    rng = np.random.default_rng(0)
    rp, cl = random_pattern(rng, 40, 55)
    s_dst = rng.standard_normal(40).astype(np.float32) * 2
    s_src = rng.standard_normal(55).astype(np.float32) * 2
    for slope in (0.2, 1.0, 0.0):
        a = oracle.edge_softmax_fwd(rp, cl, s_dst, s_src, slope)
        for v in range(40):
            e = slice(rp[v], rp[v + 1])
            raw = s_dst[v].astype(np.float64) + s_src[cl[e]].astype(np.float64)
            ref = softmax(np.where(raw > 0, raw, slope * raw))
            assert np.allclose(a[e], ref, rtol=1e-6, atol=1e-12), (slope, v)
            assert abs(a[e].astype(np.float64).sum() - 1) < 1e-6
    # equal scores: alpha = 1 / (entries of the row); slope 1 makes the score linear, so a
    # constant added to s_dst changes nothing
    a = oracle.edge_softmax_fwd(rp, cl, np.zeros(40, np.float32), np.zeros(55, np.float32), 0.2)
    assert np.allclose(a, np.repeat(1.0 / np.diff(rp), np.diff(rp)))
    a1 = oracle.edge_softmax_fwd(rp, cl, s_dst, s_src, 1.0)
    a2 = oracle.edge_softmax_fwd(rp, cl, s_dst + np.float32(3), s_src, 1.0)
    assert np.allclose(a1, a2, rtol=1e-5)
    # a score 100 above the rest takes all the weight
    s_big = s_src.copy(); s_big[cl[rp[3]]] = 100.0
    a = oracle.edge_softmax_fwd(rp, cl, s_dst, s_big, 0.2)
    assert a[rp[3]] > 1 - 1e-6


def test_sddmm_and_sums_against_dense(oracle):
    rng = np.random.default_rng(1)
    rp, cl = random_pattern(rng, 30, 47)
    F = 9
    A = rng.standard_normal((30, F + 2)).astype(np.float32)          # leading dimension > F
    B = rng.standard_normal((47, F + 1)).astype(np.float32)
    out, S = oracle.sddmm(rp, cl, A, B, F, want_S=True)
    dense = A[:, :F].astype(np.float64) @ B[:, :F].astype(np.float64).T
    rows = np.repeat(np.arange(30), np.diff(rp))
    assert np.allclose(out, dense[rows, cl], rtol=1e-6, atol=1e-7)
    assert np.all(S >= np.abs(out) - 1e-6)
    vals = rng.standard_normal(rp[-1]).astype(np.float32)
    M = sp.csr_matrix((vals.astype(np.float64), cl, rp), shape=(30, 47))
    assert np.allclose(oracle.segment_sum(rp, vals), np.asarray(M.sum(1)).ravel(), rtol=1e-6, atol=1e-6)
    assert np.allclose(oracle.column_sum(rp, cl, 47, vals), np.asarray(M.sum(0)).ravel(), rtol=1e-6, atol=1e-6)
    X = rng.standard_normal((12, F + 3)).astype(np.float32)
    X0 = X.copy()
    s = rng.standard_normal(12).astype(np.float32); a = rng.standard_normal(F).astype(np.float32)
    oracle.rank1_add(X, 10, s, a)
    assert np.array_equal(X[:10, :F], X0[:10, :F] + s[:10, None] * a[None, :])
    assert np.array_equal(X[10:], X0[10:]) and np.array_equal(X[:, F:], X0[:, F:])
    assert np.allclose(oracle.row_dot(B, a), B[:, :F].astype(np.float64) @ a, rtol=1e-6, atol=1e-6)


def test_edge_softmax_backward_against_autograd(oracle):
    rng = np.random.default_rng(2)
    n, m = 25, 33
    rp, cl = random_pattern(rng, n, m)
    rows = np.repeat(np.arange(n), np.diff(rp))
    s_dst = rng.standard_normal(n).astype(np.float32)
    s_src = rng.standard_normal(m).astype(np.float32)
    dalpha = rng.standard_normal(rp[-1]).astype(np.float32)
    slope = 0.2
    alpha = oracle.edge_softmax_fwd(rp, cl, s_dst, s_src, slope)
    de, S = oracle.edge_softmax_bwd(rp, cl, alpha, dalpha, s_dst, s_src, slope, want_S=True)
    sd = torch.tensor(s_dst, dtype=torch.float64, requires_grad=True)
    ss = torch.tensor(s_src, dtype=torch.float64, requires_grad=True)
    raw = sd[:, None] + ss[None, :]
    mask = torch.zeros(n, m, dtype=torch.bool); mask[rows, cl] = True
    e = torch.nn.functional.leaky_relu(raw, slope).masked_fill(~mask, -float("inf"))
    al = torch.softmax(e, dim=1)
    w = torch.zeros(n, m, dtype=torch.float64); w[rows, cl] = torch.tensor(dalpha, dtype=torch.float64)
    (al * w).sum().backward()
    assert np.allclose(alpha, al.detach().numpy()[rows, cl], rtol=1e-6)
    assert np.allclose(oracle.segment_sum(rp, de), sd.grad.numpy(), rtol=1e-4, atol=1e-6)
    assert np.allclose(oracle.column_sum(rp, cl, m, de), ss.grad.numpy(), rtol=1e-4, atol=1e-6)
    assert np.all(S >= np.abs(de) - 1e-7)


def _gat_loss(parts, W, att, heads):
    OL.forward_gat(parts, W, att, heads, 0.2, 1, "fp32")
    return sum(float((p.H[-1].astype(np.float64) * p.J).sum()) for p in parts)


@pytest.mark.parametrize("heads", [1, 2])
def test_gat_layer_loop_finite_differences(oracle, heads):
    """L = sum <H^(L), J> through two attention layers on two real partitions with an exact
    exchange: dW, da_dst, da_src and J^(0) (including rows that are the peer's halo rows)."""
    spec = scaled(CONFIGS["tiny"], 120, 6.0)
    spec = type(spec)(**{**spec.__dict__, "dims": (6, 4, 4), "all_parts": True, "n_parts": 2, "model": "gcn"})
    wl = build_workload(spec)
    parts = to_partdata(wl)
    W = [np_c(w).copy() for w in wl.W]
    rng = np.random.default_rng(3)
    att = [(rng.standard_normal(w.shape[1]).astype(np.float32), rng.standard_normal(w.shape[1]).astype(np.float32))
           for w in W]
    _gat_loss(parts, W, att, heads)
    OL.backward_gat(parts, W, att, heads, 0.2, 1, "fp32", exchange_first_layer=True)
    G = [sum(p.G[l] for p in parts) for l in range(1, len(W) + 1)]
    Ga = [(sum(p.Gatt[l][0] for p in parts), sum(p.Gatt[l][1] for p in parts)) for l in range(1, len(W) + 1)]
    J0 = [p.Jin[0].copy() for p in parts]
    eps = 3e-4            # small enough not to cross a ReLU / leaky-ReLU kink on these inputs

    def fd_of(arr, idx):
        old = arr[idx]
        hi, lo = np.float32(old + eps), np.float32(old - eps)
        arr[idx] = hi
        lp = _gat_loss(parts, W, att, heads)
        arr[idx] = lo
        lm = _gat_loss(parts, W, att, heads)
        arr[idx] = old
        return (lp - lm) / (float(hi) - float(lo))

    for l, w in enumerate(W):
        for _ in range(5):
            i, j = int(rng.integers(0, w.shape[0])), int(rng.integers(0, w.shape[1]))
            fd = fd_of(w, (i, j))
            assert abs(fd - G[l][i, j]) <= 3e-2 * max(abs(fd), abs(G[l][i, j]), 1e-4), ("W", l, i, j)
        for which in (0, 1):
            for _ in range(3):
                j = int(rng.integers(0, w.shape[1]))
                fd = fd_of(att[l][which], j)
                g = Ga[l][which][j]
                assert abs(fd - g) <= 3e-2 * max(abs(fd), abs(g), 1e-4), ("a", l, which, j)
    for pi, p in enumerate(parts):
        for _ in range(5):
            i, j = int(rng.integers(0, p.n_in)), int(rng.integers(0, p.X.shape[1]))
            fd = fd_of(p.X, (i, j))
            assert abs(fd - J0[pi][i, j]) <= 3e-2 * max(abs(fd), abs(J0[pi][i, j]), 1e-6), ("X", pi, i, j)
