"""Full-size GPU parity of the rows built after the 1-bit hot path: the b-bit / binary16
Low-bit kernels, the loss kernel and pipeline mode, at the sizes of the "stress" workload
(2.5 M inner rows, 2.88 M wire rows, d = 256) and in the launch shapes bench.py times.
Sampled windows / rows are recomputed by the oracle from the GPU's own inputs; integer and
bit results must match exactly, float results to the tolerances of the small-size tests."""
import numpy as np
import pytest
import torch

from oracle import layers as OL
from synth import CONFIGS, build_workload
from util import np_c

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
D = 256


def bits32(a):
    return np.ascontiguousarray(a).view(np.uint32)


def windows(n, width=300):
    mid = (n // 2) // 4 * 4 + 1
    return [(0, width), (mid, mid + width), (n - width - 3, n)]


@pytest.fixture(scope="module")
def exchange():
    """The stress partition's halo exchange: send list (mirror) into a heavy-tailed matrix."""
    wl = build_workload(CONFIGS["stress"], device=DEV)
    p = wl.parts[0]
    out = {"wl": wl, "n_in": p.n_in, "n": p.n_halo, "idx": wl.mirror.contiguous(), "X": wl.X[0]}
    yield out
    del out, wl
    torch.cuda.empty_cache()


@pytest.mark.parametrize("bits", [2, 4, 8, 16])
def test_bbit_exchange_at_full_size(oracle, exchange, bits):
    from paper_2303_01277_amd import binding as B
    from paper_2303_01277_amd import graph_engine as GE
    X, idx, n, n_in = exchange["X"], exchange["idx"], exchange["n"], exchange["n_in"]
    W1 = B.sylvie_wire_row_words_bits(D, bits)
    wire = torch.empty(n * W1, dtype=torch.int64, device=DEV)
    seed, stream = 0xFACE + bits, 4
    B.sylvie_quantize_bbit_fwd(X, D, D, idx, 0, n, bits, seed, stream, wire)
    halo = torch.full((n, D), float("nan"), device=DEV)
    B.sylvie_dequantize_bbit_fwd(wire, n, D, bits, halo, D, 0)
    torch.cuda.synchronize()
    wv = wire.view(n, W1)
    for a, b in windows(n):
        src = np_c(X[idx[a:b].long()])
        got = np_c(wv[a:b]).view(np.uint64)
        want = np.empty((b - a, D), np.float32)
        if bits == 16:
            ref = oracle.convert_fp16(src, D, b - a)
            assert np.array_equal(got.view(np.uint16), ref), (bits, a)
            oracle.recover_fp16_fwd(ref, D, want, 0)
        else:
            pk, sc, zp = oracle.quantize_bbit(src, D, b - a, bits, seed, stream, wire_row0=a)
            assert np.array_equal(got[:, :-1], pk), (bits, a)
            meta = np.ascontiguousarray(got[:, -1])
            assert np.array_equal((meta & np.uint64(0xFFFFFFFF)).astype(np.uint32), bits32(sc))
            assert np.array_equal((meta >> np.uint64(32)).astype(np.uint32), bits32(zp))
            oracle.dequantize_bbit_fwd(pk, sc, zp, D, bits, want, 0)
        assert np.array_equal(bits32(np_c(halo[a:b])), bits32(want)), (bits, a)
    # backward direction: contiguous block in, scatter-add out; sampled destination rows
    B.sylvie_quantize_bbit_bwd(halo, D, D, None, 0, n, bits, seed + 1, stream + 1, wire)
    J = torch.randn(n_in, D, device=DEV)
    J0 = J.clone()
    sp, sr, di = GE.scatter_segments(idx)
    B.sylvie_dequantize_bbit_bwd(wire, n, D, bits, J, D, sp, sr, int(di.numel()), di)
    torch.cuda.synchronize()
    rng = np.random.default_rng(bits)
    cnt = torch.bincount(idx.long(), minlength=n_in)
    busiest = torch.argsort(cnt, descending=True)[:8].cpu().numpy()
    rows = np.unique(np.concatenate([rng.integers(0, n_in, 200), busiest, [0, n_in - 1]]))
    rows_d = torch.from_numpy(rows).to(DEV)
    sel = torch.isin(idx.long(), rows_d).nonzero().flatten()          # wire rows that land there, ascending
    assert sel.numel() > 0
    dst = torch.searchsorted(rows_d, idx[sel].long()).to(torch.int32)
    wsel = np_c(wire.view(n, W1)[sel]).view(np.uint64)
    ref = np_c(J0[rows_d])
    if bits == 16:
        oracle.recover_fp16_bwd(np.ascontiguousarray(wsel).view(np.uint16), D, ref, np_c(dst))
    else:
        meta = np.ascontiguousarray(wsel[:, -1])
        sc = (meta & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.float32)
        zp = (meta >> np.uint64(32)).astype(np.uint32).view(np.float32)
        oracle.dequantize_bbit_bwd(np.ascontiguousarray(wsel[:, :-1]), sc, zp, D, bits, ref, np_c(dst))
    assert np.array_equal(bits32(np_c(J[rows_d])), bits32(ref)), bits
    untouched = (cnt == 0).nonzero().flatten()[:1000]
    assert torch.equal(J[untouched], J0[untouched])


def test_loss_kernel_at_full_size(oracle, exchange):
    from paper_2303_01277_amd import binding as B
    wl, n_in = exchange["wl"], exchange["n_in"]
    g = torch.Generator(device=DEV); g.manual_seed(5)
    H = torch.randn(n_in, D, generator=g, device=DEV) * 3
    y = wl.labels[0]
    count = float(int((y >= 0).sum()))
    J = torch.empty(n_in, D, device=DEV)
    rows = torch.empty(n_in, device=DEV)
    out = torch.zeros(1, dtype=torch.float64, device=DEV)
    B.sylvie_softmax_xent(H, D, n_in, D, y, count, J, D, rows, out)
    torch.cuda.synchronize()
    for a, b in windows(n_in, 500):
        loss, Jr, S = oracle.softmax_xent(np_c(H[a:b]), np_c(y[a:b]), count, want_S=True)
        got = np_c(J[a:b]).astype(np.float64)
        assert (np.abs(got - Jr) <= 1e-5 * np.maximum(S, 1e-30)).all()
        part = float(rows[a:b].double().sum())
        assert abs(part - loss) <= 1e-5 * abs(loss)
    total = float(rows.double().sum())
    assert abs(float(out[0]) - total) <= 1e-9 * abs(total)
    assert abs(total - np.log(D)) < 8.0                                  # order of magnitude of a random guess


def test_pipeline_mode_at_full_size(exchange):
    """bench.py's pipelined epochs: with nothing changed between epochs the pipelined epoch
    must reproduce the sequential one bit for bit (both streams, both wire generations)."""
    from paper_2303_01277_amd.trainer import LayerLoop
    wl = exchange["wl"]
    p0 = wl.parts[0]
    owner = [torch.zeros(p0.n_halo, dtype=torch.int32, device=DEV)]
    loop = LayerLoop(wl.parts, owner, [wl.mirror], wl.X, wl.J, wl.W, wl.spec.model, wl.spec.dims,
                     chunk=1024, exchange_first_layer=False, pipeline=True)
    st = loop.parts[0]

    def outputs():
        return [st.out.clone(), st.dHtil[1][: st.n_in].clone()] + [st.G[l].clone() for l in range(1, loop.L + 1)]

    loop.record = {}
    loop.step(77, OL.pair_seed, mode="sync")
    torch.cuda.synchronize()
    ref, rec = outputs(), dict(loop.record)
    for _ in range(2):
        loop.record = {}
        loop.step(77, OL.pair_seed, mode="async")
        torch.cuda.synchronize()
        for a, b in zip(outputs(), ref):
            assert torch.equal(a, b)
        assert loop.record.keys() == rec.keys()
        for k in rec:
            assert torch.equal(loop.record[k], rec[k]), k
    del loop, ref, rec
    torch.cuda.empty_cache()
