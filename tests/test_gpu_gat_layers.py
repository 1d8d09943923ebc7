"""GPU parity of the attention model's layer loop: end to end against the oracle's loop with an
exact exchange, and layer by layer (teacher-forced: the oracle recomputes each layer from the
GPU's own inputs to it) with the 1-bit exchange, whose wires must match bit for bit."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import layers as OL
from synth import CONFIGS, build_workload, scaled
from test_gpu_layers import SnapLoop, bits32, gpu_wire, o_dequantize, o_quantize
from test_gpu_layers import close as close_rel
from util import np_c, to_partdata

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_att(wl, seed):
    g = torch.Generator().manual_seed(seed)
    return [(torch.randn(w.shape[1], generator=g) / w.shape[1] ** 0.5,
             torch.randn(w.shape[1], generator=g) / w.shape[1] ** 0.5) for w in wl.W]


def build_attention_loop(wl, att, heads, wire, chunk=128, fused_sddmm=True):
    from paper_2303_01277_amd.trainer import AttentionLoop
    parts = wl.parts
    for p in parts:
        for f in ("rowptr", "col", "deg", "halo_gid", "halo_part", "halo_row"):
            setattr(p, f, getattr(p, f).to(DEV))
    if wl.mirror is not None:
        owner = [torch.zeros(parts[0].n_halo, dtype=torch.int32, device=DEV)]
        rows = [wl.mirror.to(DEV)]
    else:
        owner = [p.halo_part for p in parts]
        rows = [p.halo_row for p in parts]
    return AttentionLoop(parts, owner, rows, [x.to(DEV) for x in wl.X], [j.to(DEV) for j in wl.J],
                         [w.to(DEV) for w in wl.W], [(a.to(DEV), b.to(DEV)) for a, b in att],
                         wl.spec.dims, heads=heads, chunk=chunk, exchange_first_layer=True, wire=wire,
                         fused_sddmm=fused_sddmm)


def rel(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def workload(cfg, n_nodes):
    spec = CONFIGS[cfg] if n_nodes is None else scaled(CONFIGS[cfg], n_nodes)
    return build_workload(dataclasses.replace(spec, model="gcn"))


@pytest.mark.parametrize("heads", [1, 4])
@pytest.mark.parametrize("cfg,n_nodes", [("tiny", None), ("citation", 8_000)])
def test_attention_loop_end_to_end_exact_exchange(oracle, cfg, n_nodes, heads):
    wl = workload(cfg, n_nodes)
    att = make_att(wl, 3)
    pd = to_partdata(wl)
    W = [np_c(w) for w in wl.W]
    att_np = [(np_c(a), np_c(b)) for a, b in att]
    OL.forward_gat(pd, W, att_np, heads, 0.2, 1, "fp32")
    OL.backward_gat(pd, W, att_np, heads, 0.2, 1, "fp32", exchange_first_layer=True)
    loop = build_attention_loop(wl, att, heads, "fp32")
    loop.forward(1)
    loop.backward(1)
    torch.cuda.synchronize()
    for st, p in zip(loop.parts, pd):
        assert rel(np_c(st.out), p.H[-1]) < 5e-5
        assert rel(np_c(st.dHtil[0][: st.n_in]), p.Jin[0]) < 1e-4
        for l in range(1, len(W) + 1):
            assert rel(np_c(st.G[l]), p.G[l]) < 1e-4, l
            assert rel(np_c(st.Ga[l][0]), p.Gatt[l][0]) < 1e-4, l
            assert rel(np_c(st.Ga[l][1]), p.Gatt[l][1]) < 1e-4, l


def check_layer(oracle, rp, cl, st, snap, l, L, ht, W, a_dst, a_src, heads, slope):
    """One attention layer, forward and backward: every step recomputed by the oracle from the
    GPU's own inputs to that step (the exponential amplifies a rounding difference in the scores,
    so nothing is chained), element by element at the op tests' tolerance."""
    K = heads
    tiny = 1.1754944e-38 / 1e-5

    def close(got, ref, S, what):
        # below the smallest normal number single precision has no relative accuracy (and the
        # GPU may flush such values to zero): the bound never goes below that number
        close_rel(got, ref, np.asarray(S, np.float64) + tiny, what)
    n_in, n_loc, h = st.n_in, ht.shape[0], W.shape[1]
    F = h // K
    P = np_c(st.P[l])
    Pr, S = oracle.transform_fwd(ht, W, False, want_S=True)
    close(P, Pr, S, ("P", l))
    Hg = np_c(st.Htil[l][:n_in] if l < L else st.out)
    heads_of = lambda t, n: np_c(t).reshape(n, K)
    sd, ss, al = heads_of(st.s_dst[l], n_in), heads_of(st.s_src[l], n_loc), heads_of(st.alpha[l], -1)
    dal, de = snap["dal"].reshape(-1, K), snap["de"].reshape(-1, K)
    ds_dst, ds_src = snap["ds_dst"].reshape(n_in, K), snap["ds_src"].reshape(n_loc, K)
    dZ, dP = snap["dZ_att"], snap["dP"]
    J = snap["J"]
    want_dZ = np.where(Hg > 0, J, np.float32(0)).astype(np.float32) if l < L else J
    assert np.array_equal(bits32(dZ), bits32(want_dZ))
    row = np.repeat(np.arange(n_in), np.diff(rp))
    for k in range(K):
        sl = slice(k * F, (k + 1) * F)
        Pk, dZk = np.ascontiguousarray(P[:, sl]), np.ascontiguousarray(dZ[:, sl])
        ak_dst, ak_src = np.ascontiguousarray(a_dst[sl]), np.ascontiguousarray(a_src[sl])
        c = lambda x: np.ascontiguousarray(x[:, k])
        close(c(sd), oracle.row_dot(Pk, ak_dst, n=n_in), np.abs(Pk[:n_in].astype(np.float64)) @ np.abs(ak_dst),
              ("s_dst", l, k))
        close(c(ss), oracle.row_dot(Pk, ak_src), np.abs(Pk.astype(np.float64)) @ np.abs(ak_src), ("s_src", l, k))
        ref = oracle.edge_softmax_fwd(rp, cl, c(sd), c(ss), slope)
        # relative to alpha itself.  The score x, and x - max, are single-precision results on
        # the GPU and sit in an exponent, so their rounding (half an ulp of |x|, |max| and
        # |x - max| each, twice for the two operations that form x) is a RELATIVE error of alpha:
        # it is added to the tolerance entry by entry.  Results below the smallest normal number
        # are flushed to zero on the GPU.
        raw = c(sd).astype(np.float64)[row] + c(ss).astype(np.float64)[cl]
        x = np.where(raw > 0, raw, slope * raw)
        mx = np.maximum.reduceat(x, rp[:-1])[row]
        amp = 2.0 ** -23 * (np.abs(x) + np.abs(mx) + np.abs(x - mx))
        close(c(al), ref, ref * (1 + amp / 1e-5), ("alpha", l, k))
        # a weight below the smallest normal number counts as zero on the GPU: each entry may
        # lose that much times the gathered element
        ones = np.ones(rp[-1], np.float32)
        Z, S = oracle.aggregate_fwd(rp, cl, c(al), Pk, F, want_S=True)
        S = S + tiny * oracle.aggregate_fwd(rp, cl, ones, Pk, F, want_S=True)[1]
        close(Hg[:, sl], np.maximum(Z, 0) if l < L else Z, S, ("Z", l, k))
        ref, S = oracle.sddmm(rp, cl, dZk, Pk, F, want_S=True)
        close(c(dal), ref, S, ("dalpha", l, k))
        ref, S = oracle.edge_softmax_bwd(rp, cl, c(al), c(dal), c(sd), c(ss), slope, want_S=True)
        close(c(de), ref, S, ("de", l, k))
        ref, S = oracle.segment_sum(rp, c(de), want_S=True)
        close(c(ds_dst), ref, S, ("ds_dst", l, k))
        ref, S = oracle.column_sum(rp, cl, n_loc, c(de), want_S=True)
        close(c(ds_src), ref, S, ("ds_src", l, k))
        agg, S = oracle.aggregate_bwd(rp, cl, c(al), n_loc, dZk, F, want_S=True)
        S = S + tiny * oracle.aggregate_bwd(rp, cl, ones, n_loc, dZk, F, want_S=True)[1]
        t1 = c(ds_src).astype(np.float64)[:, None] * ak_src.astype(np.float64)[None, :]
        t2 = np.zeros_like(t1)
        t2[:n_in] = c(ds_dst).astype(np.float64)[:, None] * ak_dst.astype(np.float64)[None, :]
        close(dP[:, sl], agg.astype(np.float64) + t1 + t2, S + np.abs(t1) + np.abs(t2), ("dP", l, k))
        P64 = Pk.astype(np.float64)
        close(np_c(st.Ga[l][0][sl]), P64[:n_in].T @ c(ds_dst).astype(np.float64),
              np.abs(P64[:n_in]).T @ np.abs(c(ds_dst)).astype(np.float64), ("da_dst", l, k))
        close(np_c(st.Ga[l][1][sl]), P64.T @ c(ds_src).astype(np.float64),
              np.abs(P64).T @ np.abs(c(ds_src)).astype(np.float64), ("da_src", l, k))
    r = oracle.transform_bwd(ht, W, False, dP, dP, want_S=True)
    close(np_c(st.G[l]), r["G"], r["SG"], ("G", l))
    close(snap["dHtil_pre"], r["dA1"], r["SdA1"], ("dHtil", l))


@pytest.mark.parametrize("heads,wire", [(1, "1bit"), (2, "1bit"), (2, "4bit"), (4, "1bit"), (8, "1bit")])
@pytest.mark.parametrize("fused_sddmm", [True, False])
@pytest.mark.parametrize("cfg,n_nodes", [("tiny", None), ("stress", 12_000)])
def test_attention_loop_teacher_forced(oracle, cfg, n_nodes, heads, wire, fused_sddmm):
    """fused_sddmm: the transposed aggregation also forms the sampled product (shapes that have
    such a launch: all but tiny's 8 heads of 8 columns); otherwise the separate call."""
    wl = workload(cfg, n_nodes)
    att = make_att(wl, 5)
    pdata = to_partdata(wl)
    for pd in pdata:
        OL.build_operator(pd, "gat")
    loop = build_attention_loop(wl, att, heads, wire, fused_sddmm=fused_sddmm)
    assert not any(loop.fused_sddmm) if not fused_sddmm else \
        all(loop.fused_sddmm[1:]) == (loop.dims[1] // heads >= 16)
    bits = loop.bits
    loop.record = {}
    seed = 0x6A7
    loop.forward(seed, OL.pair_seed)
    torch.cuda.synchronize()
    snaps = SnapLoop.run(loop, seed)
    W = [np_c(w) for w in wl.W]
    L = len(W)
    for l in range(L, 0, -1):
        d, h = loop.dims[l - 1], loop.dims[l]
        a_dst, a_src = np_c(att[l - 1][0]), np_c(att[l - 1][1])
        for me, (st, pd) in enumerate(zip(loop.parts, pdata)):
            rp, cl, _ = pd.op
            ht = np_c(st.Htil[l - 1])
            # forward exchange: wires from the owners' rows, halo block recovered from them
            for b in st.blocks:
                n = b.j1 - b.j0
                src = np_c(loop.parts[b.owner].Htil[l - 1])
                ref = o_quantize(oracle, bits, src, d, n, OL.pair_seed(seed, b.owner, me), 2 * l, idx=np_c(b.rows))
                assert np.array_equal(gpu_wire(loop, ("fwd", l, me, b.j0), n, d, bits), ref)
                want = np.empty((n, d), np.float32)
                o_dequantize(oracle, bits, ref, d, want, row_offset=0)
                assert np.array_equal(bits32(ht[st.n_in + b.j0: st.n_in + b.j1]), bits32(want))
            check_layer(oracle, rp, cl, st, snaps[(l, me)], l, L, ht, W[l - 1], a_dst, a_src, heads, 0.2)
        # backward exchange: wires from the GPU's halo gradients, accumulate bit for bit
        for q, stq in enumerate(loop.parts):
            want = snaps[(l, q)]["dHtil_pre"][: stq.n_in].copy()
            for me, st in enumerate(loop.parts):
                gpre = snaps[(l, me)]["dHtil_pre"]
                for b in st.blocks:
                    if b.owner != q:
                        continue
                    n = b.j1 - b.j0
                    ref = o_quantize(oracle, bits, gpre, d, n, OL.pair_seed(seed, me, q), 2 * l + 1,
                                     row_offset=st.n_in + b.j0)
                    assert np.array_equal(gpu_wire(loop, ("bwd", l, me, b.j0), n, d, bits), ref)
                    o_dequantize(oracle, bits, ref, d, want, dst_row=np_c(b.rows))
            assert np.array_equal(bits32(np_c(stq.dHtil[l - 1][: stq.n_in])), bits32(want))


@pytest.mark.parametrize("heads", [1, 2])
def test_attention_training_reduces_the_loss_like_the_oracle(oracle, heads):
    """Exact exchange (no rounding randomness): GPU and oracle train the attention model
    independently for six epochs — loss, J^(L), backward, gradient sums over the two partitions,
    SGD on the weights and on the attention vectors; the losses agree and fall."""
    wl = workload("tiny", None)
    att = make_att(wl, 11)
    labels = [np_c(y) for y in wl.labels]
    count = float(sum(int((y >= 0).sum()) for y in labels))
    pd = to_partdata(wl)
    W = [np_c(w).copy() for w in wl.W]
    att_np = [(np_c(a).copy(), np_c(b).copy()) for a, b in att]
    eta = 1.0
    ref = []
    for e in range(6):
        OL.forward_gat(pd, W, att_np, heads, 0.2, e, "fp32")
        ref.append(OL.loss_and_gradient(pd, labels, count))
        OL.backward_gat(pd, W, att_np, heads, 0.2, e, "fp32", exchange_first_layer=False)
        OL.update_weights(pd, W, eta)
        for l in range(1, len(W) + 1):
            for i in (0, 1):
                g = oracle.sum_gradients([np.ascontiguousarray(p.Gatt[l][i]) for p in pd])
                oracle.sgd_update(att_np[l - 1][i], g, eta)
    loop = build_attention_loop(wl, att, heads, "fp32")
    loop.exchange_first_layer = False
    lab_d = [y.to(DEV) for y in wl.labels]
    got = []
    for e in range(6):
        got.append(float(loop.train_step(e, lab_d, count, eta).sum()))
    torch.cuda.synchronize()
    assert all(b < a for a, b in zip(got, got[1:])), got
    assert np.allclose(got, ref, rtol=5e-5, atol=0), (got, ref)
    for w, wr in zip(loop.W, W):
        assert np.abs(np_c(w) - wr).max() <= 1e-4 * np.abs(wr).max()
    for (a, b), (ar, br) in zip(loop.att, att_np):
        assert np.abs(np_c(a) - ar).max() <= 1e-4 * np.abs(ar).max()
        assert np.abs(np_c(b) - br).max() <= 1e-4 * np.abs(br).max()
