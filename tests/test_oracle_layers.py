"""Pins for the oracle's dense transform and the layer loop (Alg. 1 / Alg. 2)."""
import numpy as np

from synth import CONFIGS, build_workload, scaled
from oracle import layers as OL
from util import np_c, to_partdata


def test_transform_vs_numpy(oracle):
    rng = np.random.default_rng(0)
    n, k1, k2, h = 50, 13, 9, 21
    A1 = rng.standard_normal((n, k1)).astype(np.float32)
    A2 = rng.standard_normal((n, k2)).astype(np.float32)
    W = rng.standard_normal((k1 + k2, h)).astype(np.float32)
    J = rng.standard_normal((n, h)).astype(np.float32)
    A = np.concatenate([A1, A2], 1).astype(np.float64)
    P = A @ W.astype(np.float64)
    H, S = oracle.transform_fwd(A1, W, True, A2=A2, want_S=True)
    assert np.array_equal(H, np.maximum(P, 0).astype(np.float32))
    assert np.allclose(S, np.abs(A) @ np.abs(W.astype(np.float64)), rtol=1e-6)
    Hlin = oracle.transform_fwd(A1, W[:k1], False)
    assert np.array_equal(Hlin, (A1.astype(np.float64) @ W[:k1].astype(np.float64)).astype(
        np.float32))
    r = oracle.transform_bwd(A1, W, True, H, J, A2=A2, want_S=True)
    M = J.astype(np.float64) * (P.astype(np.float32) > 0)
    assert np.allclose(r["G"], A.T @ M, rtol=0, atol=1e-6 * np.abs(A.T @ M).max())
    dA = M @ W.astype(np.float64).T
    assert np.allclose(r["dA1"], dA[:, :k1], rtol=0, atol=1e-6 * np.abs(dA).max())
    assert np.allclose(r["dA2"], dA[:, k1:], rtol=0, atol=1e-6 * np.abs(dA).max())
    assert r["SG"].shape == (k1 + k2, h) and (r["SG"] >= np.abs(r["G"]) * (1 - 1e-6)).all()
    r2 = oracle.transform_bwd(A1, W[:k1], False, Hlin, J)
    assert np.allclose(r2["G"], A1.astype(np.float64).T @ J, atol=1e-5)
    assert r2["dA2"] is None


def _loss_and_grads(parts, model, W, wire):
    OL.forward(parts, model, W, seed=1, wire=wire)
    loss = sum(float((p.H[-1].astype(np.float64) * p.J).sum()) for p in parts)
    OL.backward(parts, model, W, seed=1, wire=wire, exchange_first_layer=True)
    return loss


def _check_fd(model, cfg, n_nodes):
    """Central finite differences of L = sum <H^(L), J> against the oracle's backward,
    exchange in fp32 pass-through (the quantiser is never differentiated through)."""
    spec = scaled(CONFIGS[cfg], n_nodes, 6.0)
    spec = type(spec)(**{**spec.__dict__, "dims": (6, 5, 4), "all_parts": True, "n_parts": 2, "model": model})
    wl = build_workload(spec)
    parts = to_partdata(wl)
    W = [np_c(w) for w in wl.W]
    _loss_and_grads(parts, model, W, "fp32")
    G = [sum(p.G[l] for p in parts) for l in range(1, len(W) + 1)]
    J0 = [p.Jin[0].copy() for p in parts]
    rng = np.random.default_rng(0)
    eps = 1e-3
    # weight gradients
    for l, w in enumerate(W):
        for _ in range(6):
            i, j = rng.integers(0, w.shape[0]), rng.integers(0, w.shape[1])
            old = w[i, j]
            wp, wm = np.float32(old + eps), np.float32(old - eps)
            w[i, j] = wp
            OL.forward(parts, model, W, 1, "fp32")
            lp = sum(float((p.H[-1].astype(np.float64) * p.J).sum()) for p in parts)
            w[i, j] = wm
            OL.forward(parts, model, W, 1, "fp32")
            lm = sum(float((p.H[-1].astype(np.float64) * p.J).sum()) for p in parts)
            w[i, j] = old
            fd = (lp - lm) / (float(wp) - float(wm))
            assert abs(fd - G[l][i, j]) <= 2e-2 * max(abs(fd), abs(G[l][i, j]), 1e-4), (l, i, j)
    # input-feature gradients J^(0), including rows that are halo rows of the peer
    for pi, p in enumerate(parts):
        for _ in range(6):
            i, j = rng.integers(0, p.n_in), rng.integers(0, p.X.shape[1])
            old = p.X[i, j]
            xp, xm = np.float32(old + eps), np.float32(old - eps)
            p.X[i, j] = xp
            OL.forward(parts, model, W, 1, "fp32")
            lp = sum(float((q.H[-1].astype(np.float64) * q.J).sum()) for q in parts)
            p.X[i, j] = xm
            OL.forward(parts, model, W, 1, "fp32")
            lm = sum(float((q.H[-1].astype(np.float64) * q.J).sum()) for q in parts)
            p.X[i, j] = old
            fd = (lp - lm) / (float(xp) - float(xm))
            assert abs(fd - J0[pi][i, j]) <= 3e-2 * max(abs(fd), abs(J0[pi][i, j]), 1e-6), (pi, i, j)


def test_finite_differences_gcn(oracle):
    _check_fd("gcn", "tiny", 120)


def test_finite_differences_sage(oracle):
    _check_fd("sage", "tiny", 120)


def test_partitioned_equals_whole_graph(oracle):
    """With an exact (fp32) exchange the two halves reproduce the unpartitioned layer:
    the reason full-graph training with boundary exchange is exact (Sec. 2.2)."""
    spec = scaled(CONFIGS["tiny"], 400, 8.0)
    wl2 = build_workload(spec)                                   # two real partitions
    one = type(spec)(**{**spec.__dict__, "n_parts": 1})
    wl1 = build_workload(one)
    assert wl1.parts[0].n_halo == 0 and wl1.parts[0].n_in == 400
    W = [np_c(w) for w in wl2.W]
    parts2 = to_partdata(wl2)
    parts1 = to_partdata(wl1)
    # same features / upstream gradient on both sides
    X = np.concatenate([p.X for p in parts2])
    J = np.concatenate([p.J for p in parts2])
    parts1[0].X, parts1[0].J = X, J
    for model in ("gcn", "sage"):
        Wm = W if model == "gcn" else [np.concatenate([w, w[::-1]]) for w in W]
        for p in parts1 + parts2:
            p.op = None
        OL.forward(parts1, model, Wm, 3, "fp32")
        OL.forward(parts2, model, Wm, 3, "fp32")
        H2 = np.concatenate([p.H[-1] for p in parts2])
        assert np.abs(H2 - parts1[0].H[-1]).max() <= 2e-6 * np.abs(H2).max()
        OL.backward(parts1, model, Wm, 3, "fp32", exchange_first_layer=True)
        OL.backward(parts2, model, Wm, 3, "fp32", exchange_first_layer=True)
        J2 = np.concatenate([p.Jin[0] for p in parts2])
        assert np.abs(J2 - parts1[0].Jin[0]).max() <= 2e-6 * np.abs(J2).max()
        G2 = sum(p.G[1] for p in parts2)
        assert np.abs(G2 - parts1[0].G[1]).max() <= 2e-6 * np.abs(G2).max()


def test_one_bit_loop_runs_and_is_unbiased_in_the_mean(oracle):
    """1-bit exchange on the tiny workload: halo rows take two levels per row, and the
    aggregated output averaged over seeds approaches the exact-exchange output."""
    spec = scaled(CONFIGS["tiny"], 600, 8.0)
    wl = build_workload(spec)
    W = [np_c(w) for w in wl.W]
    parts = to_partdata(wl)
    OL.forward(parts, "gcn", W, 0, "fp32")
    exact = parts[0].Z[0].astype(np.float64).copy()
    acc = np.zeros_like(exact)
    S = 60
    for seed in range(S):
        OL.forward(parts, "gcn", W, seed, "1bit")
        acc += parts[0].Z[0]
        halo = parts[0].Htil[0][parts[0].n_in:]
        assert all(len(np.unique(r)) <= 2 for r in halo[:50])
    err_mean = np.abs(acc / S - exact).mean()
    OL.forward(parts, "gcn", W, 12345, "1bit")
    err_one = np.abs(parts[0].Z[0] - exact).mean()
    assert err_mean < err_one * 2.5 / np.sqrt(S) + 1e-7
    OL.backward(parts, "gcn", W, 0, "1bit", exchange_first_layer=True)
    assert parts[0].Jin[0].shape == parts[0].X.shape and np.isfinite(parts[0].Jin[0]).all()


def test_more_bits_less_exchange_error(oracle):
    """Bit-width study (Sec. 4.3): against the full-precision exchange, the error that the
    wire adds to the layer outputs and to the propagated gradients shrinks as the wire gets
    wider: 1 > 2 > 4 > 8 bits > half precision."""
    import numpy as np
    from oracle import layers as OL
    from synth import CONFIGS, build_workload
    from util import np_c, to_partdata
    wl = build_workload(CONFIGS["tiny"])
    W = [np_c(w) for w in wl.W]

    def run(wire):
        pd = to_partdata(wl)
        OL.forward(pd, wl.spec.model, W, 7, wire)
        OL.backward(pd, wl.spec.model, W, 7, wire, exchange_first_layer=True)
        return (np.concatenate([p.H[-1].ravel() for p in pd]).astype(np.float64),
                np.concatenate([p.Jin[0].ravel() for p in pd]).astype(np.float64))

    ref_h, ref_j = run("fp32")
    errs_h, errs_j = [], []
    for wire in ("1bit", "2bit", "4bit", "8bit", "fp16"):
        h, j = run(wire)
        errs_h.append(np.linalg.norm(h - ref_h) / np.linalg.norm(ref_h))
        errs_j.append(np.linalg.norm(j - ref_j) / np.linalg.norm(ref_j))
    assert all(a > 1.5 * b for a, b in zip(errs_h, errs_h[1:])), errs_h
    assert all(a > 1.5 * b for a, b in zip(errs_j, errs_j[1:])), errs_j
    assert errs_h[-1] < 1e-3 and errs_j[-1] < 1e-3


def test_pipeline_epoch_uses_previous_wires(oracle):
    """Sylvie-A (Sec. 3.3): an epoch that computes with the previous epoch's wires.  With
    nothing changed between the two epochs (same inputs, weights and seed) the previous
    wires equal the current ones, so the pipelined epoch must reproduce the sequential one
    bit for bit; with a new seed only layer 1's wires can be predicted (its input is X) and
    the outputs must be those of a sequential epoch run on the OLD seed's halo data."""
    import numpy as np
    from oracle import layers as OL
    from synth import CONFIGS, build_workload, scaled
    from util import np_c, to_partdata
    wl = build_workload(scaled(CONFIGS["co_purchase"], 6000))
    W = [np_c(w) for w in wl.W]
    model = wl.spec.model

    def epoch(seed, prev):
        pd = to_partdata(wl)
        keep = {}
        OL.forward(pd, model, W, seed, "1bit", prev=prev, keep=keep)
        OL.backward(pd, model, W, seed, "1bit", exchange_first_layer=True, prev=prev, keep=keep)
        return pd, keep

    a, wa = epoch(5, None)
    b, wb = epoch(5, wa)                       # pipelined, nothing changed
    assert wa.keys() == wb.keys() and any(k[0] == "bwd" for k in wa)
    for k in wa:
        assert all(np.array_equal(x, y) for x, y in zip(wa[k], wb[k])), k
    for pa, pb in zip(a, b):
        assert np.array_equal(pa.H[-1], pb.H[-1]) and np.array_equal(pa.Jin[0], pb.Jin[0])
        for l in range(1, len(W) + 1):
            assert np.array_equal(pa.G[l], pb.G[l])
    c, wc = epoch(6, wa)                       # pipelined with a new seed
    s6, w6 = epoch(6, None)
    k1 = [k for k in wa if k[0] == "fwd" and k[1] == 1]
    for k in k1:                               # layer 1 quantizes X: same wires as sequentially
        assert all(np.array_equal(x, y) for x, y in zip(wc[k], w6[k]))
        assert not np.array_equal(wc[k][0], wa[k][0])
    for pa, pc in zip(a, c):                   # but it computed with the old wires throughout
        assert np.array_equal(pa.H[-1], pc.H[-1]) and np.array_equal(pa.Jin[0], pc.Jin[0])
