"""GPU parity at the full sizes of the workloads, in the launch configuration bench.py
times (fused forward, chunk 1024, Alg. 2's exchanges only): the whole layer loop runs
once per workload, then SAMPLED outputs of every step are recomputed by the oracle from
the GPU's own inputs to that step.  Samples always include the first and last rows, the
ragged tail of the last wavefront and the longest CSR rows (the ones cut into tasks).
Same bars as the small-size tests: wires and the backward accumulate bit-exact, float
sums within 1e-5 * max(|ref|, S)."""
import numpy as np
import pytest
import torch

from oracle import layers as OL
from synth import CONFIGS, build_workload
from util import np_c, split_wire

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-5
SEED = 0xC0FFEE


def bits32(a):
    return np.ascontiguousarray(a).view(np.uint32)


def close(got, ref, S, what):
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = TOL * np.maximum(np.abs(ref), S).astype(np.float64)
    bad = err > bound
    assert not bad.any(), (what, int(bad.sum()), float((err / np.maximum(bound, 1e-300)).max()))


class Run:
    """One forward + backward pass of a workload on the GPU with what the checks need
    kept on the device: every wire, and per backward layer the gradient block before the
    exchange and the dense gradient that fed the transposed aggregation."""

    def __init__(self, name):
        from paper_2303_01277_amd import binding as B
        from paper_2303_01277_amd.trainer import LayerLoop
        spec = CONFIGS[name]
        self.spec = spec
        wl = build_workload(spec, device=DEV)
        self.wl = wl
        p0 = wl.parts[0]
        owner = [torch.zeros(p0.n_halo, dtype=torch.int32, device=DEV)]
        # the two-step backward exposes the float halo gradients the oracle is fed with;
        # the fused backward bench.py times is then required to match it bit for bit
        self.loop = LayerLoop(wl.parts, owner, [wl.mirror], wl.X, wl.J, wl.W, spec.model,
                              spec.dims, chunk=1024, exchange_first_layer=False, fused=True,
                              fused_bwd=False)
        self.loop.record = {}
        self.loop.forward(SEED, OL.pair_seed)
        self.pre = {}
        orig = B.sylvie_quantize_1bit_bwd
        loop = self.loop

        def hook(src, ld, d, idx, off, n, sd, stream_id, wire):
            l = (stream_id - 1) // 2
            st = loop.parts[0]
            self.pre[l] = {"dHtil": st.dHtil[l - 1].clone(),
                           "dZ": st.dZ.view(-1)[: st.n_in * d].view(st.n_in, d).clone(),
                           "dself": None if st.dself is None else
                           st.dself.view(-1)[: st.n_in * d].view(st.n_in, d).clone()}
            return orig(src, ld, d, idx, off, n, sd, stream_id, wire)

        B.sylvie_quantize_1bit_bwd = hook
        try:
            self.loop.backward(SEED, OL.pair_seed)
        finally:
            B.sylvie_quantize_1bit_bwd = orig
        torch.cuda.synchronize()
        self.fused = LayerLoop(wl.parts, owner, [wl.mirror], wl.X, wl.J, wl.W, spec.model,
                               spec.dims, chunk=1024, exchange_first_layer=False, fused=True,
                               fused_bwd=True)
        self.fused.record = {}
        self.fused.forward(SEED, OL.pair_seed)
        # what the fused inner-row call was given, per layer (it is called for l = L .. 2)
        self.fused_in = {}
        orig_i = B.sylvie_aggregate_csr_bwd_integrate
        L = len(spec.dims) - 1

        def hook_i(*a, **kw):
            l = L - len(self.fused_in)
            self.fused_in[l] = {"dZ": a[7].clone(), "dself": None if a[12] is None else a[12].clone()}
            return orig_i(*a, **kw)

        B.sylvie_aggregate_csr_bwd_integrate = hook_i
        try:
            self.fused.backward(SEED, OL.pair_seed)
        finally:
            B.sylvie_aggregate_csr_bwd_integrate = orig_i
        torch.cuda.synchronize()
        self.st = self.loop.parts[0]
        rp, cl, dg = np_c(p0.rowptr), np_c(p0.col), np_c(p0.deg)
        import oracle as O
        self.op = O.gcn_operator(rp, cl, dg, p0.n_in) if spec.model == "gcn" else \
            (rp, cl, O.mean_weights(rp, p0.n_in))
        self.mirror = np_c(wl.mirror)
        self.rng = np.random.default_rng(7)


@pytest.fixture(scope="module")
def run(request):
    """One GPU pass per workload, shared by the checks below (pytest groups the tests of
    one workload together and drops the pass before the next workload is built)."""
    r = Run(request.param)
    yield r
    del r
    torch.cuda.empty_cache()


WORKLOADS = ["dense_social", "co_purchase", "citation", "stress"]
allruns = pytest.mark.parametrize("run", WORKLOADS, indirect=True)


def windows(n, width=300):
    """Row windows [a, b): the start, two interior stretches, and the ragged end."""
    if n <= 4 * width:
        return [(0, n)]
    mid = (n // 2) // 4 * 4 + 1
    return [(0, width), (mid, mid + width), (n - width - 3, n)]


def sample_rows(rng, rowptr, n_rows, k=192):
    """Random rows plus the longest rows, the first and the last."""
    deg = np.diff(rowptr[: n_rows + 1])
    longest = np.argsort(deg)[-12:]
    pick = np.concatenate([rng.integers(0, n_rows, k), longest, [0, n_rows - 1]])
    return np.unique(pick).astype(np.int64)


def sub_csr(rowptr, col, w, rows):
    """CSR of the listed rows with columns renumbered to a compact range."""
    seg = [np.arange(rowptr[r], rowptr[r + 1]) for r in rows]
    lens = np.array([len(s) for s in seg])
    e = np.concatenate(seg) if len(seg) else np.zeros(0, np.int64)
    cols = col[e]
    uniq, inv = np.unique(cols, return_inverse=True)
    rp = np.zeros(len(rows) + 1, np.int64)
    rp[1:] = np.cumsum(lens)
    return rp, inv.astype(np.int32), np.ascontiguousarray(w[e]), uniq


@allruns
def test_forward_wires(oracle, run):
    st, dims = run.st, run.spec.dims
    for l in range(1, len(dims)):
        d = dims[l - 1]
        W1 = (d + 63) // 64 + 1
        wire = run.loop.record[("fwd", l, 0, 0)]
        src = st.Htil[l - 1]
        for a, b in windows(st.n_halo):
            idx = run.mirror[a:b]
            uniq, inv = np.unique(idx, return_inverse=True)
            rows = np_c(src[torch.from_numpy(uniq).to(DEV)])
            ref = oracle.quantize_1bit(rows, d, b - a, OL.pair_seed(SEED, 0, 0), 2 * l,
                                       idx=inv.astype(np.int32), wire_row0=a)
            pk, sc, zp = split_wire(np_c(wire[a * W1: b * W1]), b - a, d)
            assert np.array_equal(pk, ref[0]), ("bits", l, a)
            assert np.array_equal(bits32(sc), bits32(ref[1])) and \
                np.array_equal(bits32(zp), bits32(ref[2])), ("meta", l, a)


@allruns
def test_forward_aggregate_and_transform(oracle, run):
    st, dims, model = run.st, run.spec.dims, run.spec.model
    rp, cl, w = run.op
    L = len(dims) - 1
    for l in range(1, L + 1):
        d = dims[l - 1]
        W1 = (d + 63) // 64 + 1
        rows = sample_rows(run.rng, rp, st.n_in)
        srp, scol, sw, uniq = sub_csr(rp, cl, w, rows)
        inner = uniq < st.n_in
        X = np.empty((len(uniq), d), np.float32)
        X[inner] = np_c(st.Htil[l - 1][torch.from_numpy(uniq[inner]).to(DEV)])
        # halo rows: the oracle's dequantizer on the GPU's wire rows
        hj = uniq[~inner] - st.n_in
        wire = run.loop.record[("fwd", l, 0, 0)].view(-1, W1)
        pk, sc, zp = split_wire(np_c(wire[torch.from_numpy(hj).to(DEV)]), len(hj), d)
        halo = np.empty((len(hj), d), np.float32)
        oracle.dequantize_1bit_fwd(pk, sc, zp, d, halo, 0)
        X[~inner] = halo
        Z, S = oracle.aggregate_fwd(srp, scol, sw, X, d, want_S=True)
        rt = torch.from_numpy(rows).to(DEV)
        Zg = np_c(st.Z[l - 1][rt])
        close(Zg, Z, S, ("Z", l))
        Hg = np_c((st.Htil[l] if l < L else st.out)[rt])
        Wl = np_c(run.wl.W[l - 1])
        if model == "gcn":
            H, SH = oracle.transform_fwd(Zg, Wl, l != L, want_S=True)
        else:
            H, SH = oracle.transform_fwd(np_c(st.Htil[l - 1][rt]), Wl, l != L, A2=Zg, want_S=True)
        close(Hg, H, SH, ("H", l))


@allruns
def test_backward_transform(oracle, run):
    st, dims, model = run.st, run.spec.dims, run.spec.model
    L = len(dims) - 1
    for l in range(L, 0, -1):
        d, h = dims[l - 1], dims[l]
        relu = l != L
        Wl = np_c(run.wl.W[l - 1])
        Hl = st.Htil[l] if l < L else st.out
        Jl = st.J if l == L else st.dHtil[l]
        # feature gradient on sampled rows
        if l > 1:
            rt = torch.from_numpy(np.unique(run.rng.integers(0, st.n_in, 256))).to(DEV)
            A1 = np_c((st.Z[l - 1] if model == "gcn" else st.Htil[l - 1])[rt])
            A2 = None if model == "gcn" else np_c(st.Z[l - 1][rt])
            r = oracle.transform_bwd(A1, Wl, relu, np_c(Hl[rt]), np_c(Jl[rt]), A2=A2,
                                     want_G=False, want_S=True)
            if model == "gcn":
                close(np_c(run.pre[l]["dZ"][rt]), r["dA1"], r["SdA1"], ("dZ", l))
            else:
                close(np_c(run.pre[l]["dself"][rt]), r["dA1"], r["SdA1"], ("dself", l))
                close(np_c(run.pre[l]["dZ"][rt]), r["dA2"], r["SdA2"], ("dZ", l))
        # weight gradient: sampled entries G[ks, js], each a full-length sum over the rows
        K = Wl.shape[0]
        ks = np.unique(run.rng.integers(0, K, 6))
        js = np.unique(run.rng.integers(0, h, 6))
        kt, jt = torch.from_numpy(ks).to(DEV), torch.from_numpy(js).to(DEV)
        Acat = st.Z[l - 1] if model == "gcn" else None
        if model == "gcn":
            Ak = np_c(Acat[:, kt])
        else:
            left = st.Htil[l - 1][: st.n_in]
            Ak = np_c(torch.where((kt < d)[None, :], left[:, kt.clamp(max=d - 1)],
                                  st.Z[l - 1][:, (kt - d).clamp(min=0)]))
        Hs, Js = np_c(Hl[: st.n_in][:, jt]), np_c(Jl[: st.n_in][:, jt])
        r = oracle.transform_bwd(Ak, np.zeros((len(ks), len(js)), np.float32), relu, Hs, Js,
                                 want_dA=False, want_S=True)
        Gg = np_c(st.G[l])[np.ix_(ks, js)]
        close(Gg, r["G"], r["SG"], ("G", l))


@allruns
def test_backward_aggregate_and_exchange(oracle, run):
    st, dims, model = run.st, run.spec.dims, run.spec.model
    rp, cl, w = run.op
    L = len(dims) - 1
    n_loc = st.n_in + st.n_halo
    # transposed row lengths: how often each local row is referenced
    refs = np.bincount(cl, minlength=n_loc)
    for l in range(L, 1, -1):
        d = dims[l - 1]
        W1 = (d + 63) // 64 + 1
        pre = run.pre[l]
        dZ = np_c(pre["dZ"])
        hubs = np.argsort(refs)[-10:]
        sel = np.unique(np.concatenate([run.rng.integers(0, n_loc, 160), hubs,
                                        [0, st.n_in - 1, st.n_in, n_loc - 1]])).astype(np.int32)
        out, S = oracle.aggregate_bwd_rows(rp, cl, w, dZ, d, sel)
        out = out.astype(np.float64)
        st_ = torch.from_numpy(sel.astype(np.int64)).to(DEV)
        if pre["dself"] is not None:
            isin = sel < st.n_in
            ds = np_c(pre["dself"][st_[torch.from_numpy(isin).to(DEV)]])
            out[isin] += ds
            S[isin] += np.abs(ds)
        close(np_c(pre["dHtil"][st_]), out, S, ("dHtil", l))
        # wires of the halo-gradient block
        wire = run.loop.record[("bwd", l, 0, 0)]
        for a, b in windows(st.n_halo):
            rows = np_c(pre["dHtil"][st.n_in + a: st.n_in + b])
            ref = oracle.quantize_1bit(rows, d, b - a, OL.pair_seed(SEED, 0, 0), 2 * l + 1,
                                       wire_row0=a)
            pk, sc, zp = split_wire(np_c(wire[a * W1: b * W1]), b - a, d)
            assert np.array_equal(pk, ref[0]), ("bwd bits", l, a)
            assert np.array_equal(bits32(sc), bits32(ref[1])) and \
                np.array_equal(bits32(zp), bits32(ref[2])), ("bwd meta", l, a)
        # integrate: sampled destinations, all the wire rows that land on each, in order
        order = np.argsort(run.mirror, kind="stable")
        sorted_m = run.mirror[order]
        dsts = np.unique(np.concatenate([run.rng.integers(0, st.n_in, 200),
                                         np.argsort(np.bincount(run.mirror, minlength=st.n_in))[-5:]]))
        lo = np.searchsorted(sorted_m, dsts, "left")
        hi = np.searchsorted(sorted_m, dsts, "right")
        wire2 = wire.view(-1, W1)
        J = np_c(pre["dHtil"][torch.from_numpy(dsts).to(DEV)])
        for i, (a, b) in enumerate(zip(lo, hi)):
            js = order[a:b]                                   # ascending wire rows
            if len(js) == 0:
                continue
            pk, sc, zp = split_wire(np_c(wire2[torch.from_numpy(js).to(DEV)]), len(js), d)
            tgt = J[i: i + 1].copy()
            oracle.dequantize_1bit_bwd(pk, sc, zp, d, tgt, np.zeros(len(js), np.int32))
            J[i] = tgt[0]
        got = np_c(st.dHtil[l - 1][torch.from_numpy(dsts).to(DEV)])
        assert np.array_equal(bits32(got), bits32(J)), ("integrate", l)


@allruns
def test_fused_backward_matches(run):
    """bench.py's configuration (fused backward) against the two-step backward checked above."""
    a, b = run.loop, run.fused
    assert a.record.keys() == b.record.keys()
    for k in a.record:
        assert torch.equal(a.record[k], b.record[k]), k
    sa, sb = a.parts[0], b.parts[0]
    for l in range(1, len(run.spec.dims) - 1):
        assert torch.equal(sa.dHtil[l][: sa.n_in], sb.dHtil[l]), l
    for l in range(1, len(run.spec.dims)):
        assert torch.equal(sa.G[l], sb.G[l]), l
    assert torch.equal(sa.out, sb.out)


@allruns
def test_fused_integrate_against_oracle(oracle, run):
    """The inner-row call of the fused backward (transposed aggregation + received gradients
    added in its epilogue) against the oracle directly: Alg. 2's feature gradient of sampled
    inner rows from the call's own dense gradient, then the oracle's ordered accumulate of the
    wire rows that land on each.  The sum carries the float tolerance, the adds change nothing
    about it."""
    st, dims = run.fused.parts[0], run.spec.dims
    rp, cl, w = run.op
    L = len(dims) - 1
    order = np.argsort(run.mirror, kind="stable")
    sorted_m = run.mirror[order]
    refs = np.bincount(cl, minlength=st.n_in + st.n_halo)[: st.n_in]
    for l in range(L, 1, -1):
        d = dims[l - 1]
        W1 = (d + 63) // 64 + 1
        fin = run.fused_in[l]
        dZ = np_c(fin["dZ"])
        sel = np.unique(np.concatenate([
            run.rng.integers(0, st.n_in, 160), np.argsort(refs)[-8:],
            np.argsort(np.bincount(run.mirror, minlength=st.n_in))[-5:], [0, st.n_in - 1]])).astype(np.int32)
        out, S = oracle.aggregate_bwd_rows(rp, cl, w, dZ, d, sel)
        sel_t = torch.from_numpy(sel.astype(np.int64)).to(DEV)
        ref64 = out.astype(np.float64)
        if fin["dself"] is not None:
            ds = np_c(fin["dself"][sel_t])
            ref64 += ds
            S = S + np.abs(ds)
        J = ref64.astype(np.float32)
        wire2 = run.fused.record[("bwd", l, 0, 0)].view(-1, W1)
        lo = np.searchsorted(sorted_m, sel, "left")
        hi = np.searchsorted(sorted_m, sel, "right")
        for i, (a, b) in enumerate(zip(lo, hi)):
            js = order[a:b]                                   # ascending wire rows
            if len(js) == 0:
                continue
            pk, sc, zp = split_wire(np_c(wire2[torch.from_numpy(js).to(DEV)]), len(js), d)
            tgt = J[i: i + 1].copy()
            oracle.dequantize_1bit_bwd(pk, sc, zp, d, tgt, np.zeros(len(js), np.int32))
            J[i] = tgt[0]
            S[i] += (np.abs(zp) + np.abs(sc)).sum()           # magnitudes of the added levels
        close(np_c(st.dHtil[l - 1][sel_t]), J, S, ("fused integrate", l))


@allruns
def test_fused_step_repeats_bitwise(run):
    """The same step twice on the same loop object: every wire, gradient and output repeats
    bit for bit (long rows are cut into tasks and joined in task order, nothing is atomic)."""
    loop = run.fused
    st = loop.parts[0]
    first = {k: v.clone() for k, v in loop.record.items()}
    out0 = st.out.clone()
    G0 = [None if g is None else g.clone() for g in st.G]
    dH0 = [None if (g is None or l == 0) else g.clone() for l, g in enumerate(st.dHtil)]
    Z0 = [z.clone() for z in st.Z]
    loop.record = {}
    loop.forward(SEED, OL.pair_seed)
    loop.backward(SEED, OL.pair_seed)
    torch.cuda.synchronize()
    assert loop.record.keys() == first.keys()
    for k in first:
        assert torch.equal(first[k], loop.record[k]), k
    assert torch.equal(out0, st.out)
    for a, b in zip(Z0, st.Z):
        assert torch.equal(a, b)
    for a, b in zip(G0, st.G):
        assert a is None or torch.equal(a, b)
    for a, b in zip(dH0, st.dHtil):
        assert a is None or torch.equal(a, b)
