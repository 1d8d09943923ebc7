"""Oracle layer loop: Alg. 1 (forward) and Alg. 2 (backward) of Sylvie-S on the
partitions of one graph, all partitions stepped in one process and the send /
receive replaced by handing the wire arrays over (test infrastructure only).

A partition is described by plain numpy arrays (see `PartData`).  Every halo row
j of partition p names its owner partition `halo_part[j]` and the owner's inner
row `halo_row[j]`; halo rows are grouped by owner in ascending order.  A single
partition whose halo rows all name itself is the "loopback" stand-in for absent
peers.

wire = "1bit": quantize -> (packed, scale, zero) -> dequantize (Sec. 3.2).
wire = "2bit" / "4bit" / "8bit": the same with B = 2^b - 1 bins; wire = "fp16": rows
rounded to binary16 (the other points of the bit-width study, Sec. 4.3).
Sylvie-A (Sec. 3.3): with `prev` given, every layer computes with the wires of the
previous epoch found there, while this epoch's wires are still produced (and stored in
`keep`), to be used by the next epoch.  1-bit wire only.
wire = "fp32": the rows are copied unchanged (vanilla full-precision exchange,
Sec. 2.2), used where a check must not depend on the rounding randomness.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import api as O


WIRE_BITS = {"2bit": 2, "4bit": 4, "8bit": 8}


@dataclass
class PartData:
    n_in: int
    n_halo: int
    rowptr: np.ndarray          # int64 [n_in+1], adjacency without self loops
    col: np.ndarray             # int32 [nnz]
    deg: np.ndarray             # int32 [n_in+n_halo], global degrees
    halo_part: np.ndarray       # int32 [n_halo]
    halo_row: np.ndarray        # int32 [n_halo]
    X: np.ndarray               # f32 [n_in, d_0]
    J: np.ndarray               # f32 [n_in, d_L] upstream gradient
    # filled by the loop
    op: tuple = None            # (rowptr, col, w) of the normalised operator
    Htil: List[np.ndarray] = field(default_factory=list)   # Htil[l-1]: input of layer l
    Z: List[np.ndarray] = field(default_factory=list)
    H: List[np.ndarray] = field(default_factory=list)      # H[l]: output of layer l (H[0] = X)
    G: List[Optional[np.ndarray]] = field(default_factory=list)
    Jin: List[Optional[np.ndarray]] = field(default_factory=list)  # Jin[l] = J^(l)


def pair_seed(seed: int, sender: int, receiver: int) -> int:
    """One seed per ordered (sender, receiver) pair so no two wires share randomness."""
    return (int(seed) + 0x9E3779B97F4A7C15 * (sender * 4096 + receiver + 1)) & (2**64 - 1)


def owner_blocks(p: PartData):
    """[(owner, j0, j1)]: maximal runs of halo rows with the same owner."""
    out = []
    j = 0
    while j < p.n_halo:
        q = int(p.halo_part[j])
        k = j
        while k < p.n_halo and int(p.halo_part[k]) == q:
            k += 1
        out.append((q, j, k))
        j = k
    return out


def build_operator(p: PartData, model: str):
    if model == "gcn":
        p.op = O.gcn_operator(p.rowptr, p.col, p.deg, p.n_in)
    elif model == "gat":
        # attention runs over the same entries as the GCN operator (neighbours + self loop);
        # the weights of that operator are not used
        p.op = O.gcn_operator(p.rowptr, p.col, p.deg, p.n_in)
    elif model == "sage":
        p.op = (p.rowptr, p.col, O.mean_weights(p.rowptr, p.n_in))
    else:
        raise ValueError(model)


def forward(parts: List[PartData], model: str, W: List[np.ndarray], seed: int, wire="1bit",
            prev: Optional[dict] = None, keep: Optional[dict] = None):
    """Alg. 1 lines 8-17 for one epoch.  keep: dict that receives this epoch's wires under
    ("fwd", l, receiver, j0); prev: such a dict of the previous epoch, whose wires are then
    the ones dequantized into the halo block (Sylvie-A)."""
    L = len(W)
    if (prev is not None or keep is not None) and wire != "1bit":
        raise ValueError("prev / keep are for the 1-bit wire")
    for me, p in enumerate(parts):
        if p.op is None:
            build_operator(p, model)
        p.H = [p.X]
        p.Htil, p.Z = [], []
    for l in range(1, L + 1):
        d = parts[0].H[l - 1].shape[1]
        for me, p in enumerate(parts):
            ht = np.zeros((p.n_in + p.n_halo, d), np.float32)
            ht[: p.n_in] = p.H[l - 1]
            # quantize at the owner, hand over, dequantize into the halo block
            for (q, j0, j1) in owner_blocks(p):
                src = parts[q].H[l - 1]
                idx = np.ascontiguousarray(p.halo_row[j0:j1])
                if wire == "1bit":
                    pk, sc, zp = O.quantize_1bit(src, d, j1 - j0, pair_seed(seed, q, me),
                                                 2 * l + 0, idx=idx)
                    if keep is not None:
                        keep[("fwd", l, me, j0)] = (pk, sc, zp)
                    if prev is not None:
                        pk, sc, zp = prev[("fwd", l, me, j0)]
                    O.dequantize_1bit_fwd(pk, sc, zp, d, ht, p.n_in + j0)
                elif wire in WIRE_BITS:
                    b = WIRE_BITS[wire]
                    pk, sc, zp = O.quantize_bbit(src, d, j1 - j0, b, pair_seed(seed, q, me),
                                                 2 * l + 0, idx=idx)
                    O.dequantize_bbit_fwd(pk, sc, zp, d, b, ht, p.n_in + j0)
                elif wire == "fp16":
                    O.recover_fp16_fwd(O.convert_fp16(src, d, j1 - j0, idx=idx), d, ht, p.n_in + j0)
                else:
                    ht[p.n_in + j0: p.n_in + j1] = src[idx]
            p.Htil.append(ht)
        for p in parts:
            rp, cl, w = p.op
            Z = O.aggregate_fwd(rp, cl, w, p.Htil[l - 1], d)
            p.Z.append(Z)
            relu = l != L
            if model == "gcn":
                H = O.transform_fwd(Z, W[l - 1], relu)
            else:
                H = O.transform_fwd(np.ascontiguousarray(p.H[l - 1]), W[l - 1], relu, A2=Z)
            p.H.append(H)


def backward(parts: List[PartData], model: str, W: List[np.ndarray], seed: int, wire="1bit",
             exchange_first_layer=False, prev: Optional[dict] = None, keep: Optional[dict] = None):
    """Alg. 2 for one epoch (weight gradients stay per partition: no all-reduce).

    exchange_first_layer=True also computes and exchanges J^(0), as if another
    layer sat below layer 1.
    """
    L = len(W)
    for p in parts:
        p.Jin = [None] * (L + 1)
        p.G = [None] * (L + 1)
        p.Jin[L] = p.J
    for l in range(L, 0, -1):
        need_dx = l > 1 or exchange_first_layer
        dHt = []
        for p in parts:
            relu = l != L
            Z = p.Z[l - 1]
            if model == "gcn":
                r = O.transform_bwd(Z, W[l - 1], relu, p.H[l], p.Jin[l], want_dA=need_dx)
                dZ, dself = r["dA1"], None
            else:
                r = O.transform_bwd(np.ascontiguousarray(p.H[l - 1]), W[l - 1], relu, p.H[l],
                                    p.Jin[l], A2=Z, want_dA=need_dx)
                dself, dZ = r["dA1"], r["dA2"]
            p.G[l] = r["G"]
            if not need_dx:
                dHt.append(None)
                continue
            rp, cl, w = p.op
            d = dZ.shape[1]
            g = O.aggregate_bwd(rp, cl, w, p.n_in + p.n_halo, dZ, d)
            if dself is not None:
                g[: p.n_in] = g[: p.n_in] + dself
            dHt.append(g)
        if not need_dx:
            continue
        for p, g in zip(parts, dHt):
            p.Jin[l - 1] = np.ascontiguousarray(g[: p.n_in]).copy()
        for me, (p, g) in enumerate(zip(parts, dHt)):
            d = g.shape[1]
            for (q, j0, j1) in owner_blocks(p):
                dst = np.ascontiguousarray(p.halo_row[j0:j1])
                if wire == "1bit":
                    pk, sc, zp = O.quantize_1bit(g, d, j1 - j0, pair_seed(seed, me, q), 2 * l + 1,
                                                 row_offset=p.n_in + j0)
                    if keep is not None:
                        keep[("bwd", l, me, j0)] = (pk, sc, zp)
                    if prev is not None:
                        pk, sc, zp = prev[("bwd", l, me, j0)]
                    O.dequantize_1bit_bwd(pk, sc, zp, d, parts[q].Jin[l - 1], dst)
                elif wire in WIRE_BITS:
                    b = WIRE_BITS[wire]
                    pk, sc, zp = O.quantize_bbit(g, d, j1 - j0, b, pair_seed(seed, me, q),
                                                 2 * l + 1, row_offset=p.n_in + j0)
                    O.dequantize_bbit_bwd(pk, sc, zp, d, b, parts[q].Jin[l - 1], dst)
                elif wire == "fp16":
                    O.recover_fp16_bwd(O.convert_fp16(g, d, j1 - j0, row_offset=p.n_in + j0), d,
                                       parts[q].Jin[l - 1], dst)
                else:
                    np.add.at(parts[q].Jin[l - 1], dst, g[p.n_in + j0: p.n_in + j1])


def loss_and_gradient(parts: List[PartData], labels: List[np.ndarray], count: float):
    """Alg. 1 last line / Alg. 2 first line: J^(L) of every partition from its H^(L); returns
    the loss of the whole graph (sum of the partition contributions)."""
    total = 0.0
    for p, y in zip(parts, labels):
        loss, J = O.softmax_xent(np.ascontiguousarray(p.H[-1]), y, count)
        p.J = J
        total += loss
    return total


def update_weights(parts: List[PartData], W: List[np.ndarray], eta: float):
    """Alg. 2 last two lines with every partition in one process: G = sum over partitions
    (ascending), W = W - eta G, in place."""
    for l in range(1, len(W) + 1):
        G = O.sum_gradients([np.ascontiguousarray(p.G[l]) for p in parts])
        O.sgd_update(W[l - 1], G, eta)


# ---- attention model (GAT): transform first, then aggregate with learned edge weights --------

def _exchange_rows_fwd(parts, l, d, seed, wire):
    """Htilde^(l-1) of every partition: inner rows + recovered halo rows (Alg. 1 exchange)."""
    out = []
    for me, p in enumerate(parts):
        ht = np.zeros((p.n_in + p.n_halo, d), np.float32)
        ht[: p.n_in] = p.H[l - 1]
        for (q, j0, j1) in owner_blocks(p):
            src = parts[q].H[l - 1]
            idx = np.ascontiguousarray(p.halo_row[j0:j1])
            if wire == "1bit":
                pk, sc, zp = O.quantize_1bit(src, d, j1 - j0, pair_seed(seed, q, me), 2 * l + 0, idx=idx)
                O.dequantize_1bit_fwd(pk, sc, zp, d, ht, p.n_in + j0)
            elif wire in WIRE_BITS:
                b = WIRE_BITS[wire]
                pk, sc, zp = O.quantize_bbit(src, d, j1 - j0, b, pair_seed(seed, q, me), 2 * l + 0, idx=idx)
                O.dequantize_bbit_fwd(pk, sc, zp, d, b, ht, p.n_in + j0)
            elif wire == "fp16":
                O.recover_fp16_fwd(O.convert_fp16(src, d, j1 - j0, idx=idx), d, ht, p.n_in + j0)
            else:
                ht[p.n_in + j0: p.n_in + j1] = src[idx]
        out.append(ht)
    return out


def _exchange_rows_bwd(parts, dHt, l, seed, wire):
    """J^(l-1): inner rows of dHtilde plus the received halo-row gradients (Alg. 2 exchange)."""
    for p, g in zip(parts, dHt):
        p.Jin[l - 1] = np.ascontiguousarray(g[: p.n_in]).copy()
    for me, (p, g) in enumerate(zip(parts, dHt)):
        d = g.shape[1]
        for (q, j0, j1) in owner_blocks(p):
            dst = np.ascontiguousarray(p.halo_row[j0:j1])
            if wire == "1bit":
                pk, sc, zp = O.quantize_1bit(g, d, j1 - j0, pair_seed(seed, me, q), 2 * l + 1,
                                             row_offset=p.n_in + j0)
                O.dequantize_1bit_bwd(pk, sc, zp, d, parts[q].Jin[l - 1], dst)
            elif wire in WIRE_BITS:
                b = WIRE_BITS[wire]
                pk, sc, zp = O.quantize_bbit(g, d, j1 - j0, b, pair_seed(seed, me, q), 2 * l + 1,
                                             row_offset=p.n_in + j0)
                O.dequantize_bbit_bwd(pk, sc, zp, d, b, parts[q].Jin[l - 1], dst)
            elif wire == "fp16":
                O.recover_fp16_bwd(O.convert_fp16(g, d, j1 - j0, row_offset=p.n_in + j0), d,
                                   parts[q].Jin[l - 1], dst)
            else:
                np.add.at(parts[q].Jin[l - 1], dst, g[p.n_in + j0: p.n_in + j1])


def forward_gat(parts: List[PartData], W, att, heads: int, slope: float, seed: int, wire="1bit"):
    """Alg. 1 with the attention layer: P = Htilde W on inner + halo rows, per head
    alpha = softmax over each row's entries of leaky_relu(P_v . a_dst + P_u . a_src),
    Z = sum alpha P_u, H = relu(Z) except on the last layer.  att[l-1] = (a_dst, a_src),
    each of length d_l with the heads' vectors side by side."""
    L = len(W)
    for p in parts:
        if p.op is None:
            build_operator(p, "gat")
        p.H = [p.X]
        p.Htil, p.P, p.alpha, p.s_dst, p.s_src, p.Zpre = [], [], [], [], [], []
    for l in range(1, L + 1):
        d, h = W[l - 1].shape
        F = h // heads
        for p, ht in zip(parts, _exchange_rows_fwd(parts, l, d, seed, wire)):
            p.Htil.append(ht)
        for p in parts:
            rp, cl, _ = p.op
            P = O.transform_fwd(p.Htil[l - 1], W[l - 1], False)
            a_dst, a_src = att[l - 1]
            Z = np.empty((p.n_in, h), np.float32)
            al, sd, ss = [], [], []
            for k in range(heads):
                Pk = np.ascontiguousarray(P[:, k * F:(k + 1) * F])
                s_dst = O.row_dot(Pk, np.ascontiguousarray(a_dst[k * F:(k + 1) * F]), n=p.n_in)
                s_src = O.row_dot(Pk, np.ascontiguousarray(a_src[k * F:(k + 1) * F]))
                alpha = O.edge_softmax_fwd(rp, cl, s_dst, s_src, slope)
                Z[:, k * F:(k + 1) * F] = O.aggregate_fwd(rp, cl, alpha, Pk, F)
                al.append(alpha); sd.append(s_dst); ss.append(s_src)
            p.P.append(P); p.alpha.append(al); p.s_dst.append(sd); p.s_src.append(ss)
            p.Zpre.append(Z)
            p.H.append(np.maximum(Z, np.float32(0)) if l != L else Z.copy())


def backward_gat(parts: List[PartData], W, att, heads: int, slope: float, seed: int, wire="1bit",
                 exchange_first_layer=False):
    """Alg. 2 with the attention layer.  Per partition p.G[l] = dW, p.Gatt[l] = (da_dst, da_src)."""
    L = len(W)
    for p in parts:
        p.Jin = [None] * (L + 1)
        p.G = [None] * (L + 1)
        p.Gatt = [None] * (L + 1)
        p.Jin[L] = p.J
    for l in range(L, 0, -1):
        d, h = W[l - 1].shape
        F = h // heads
        need_dx = l > 1 or exchange_first_layer
        dHt = []
        for p in parts:
            rp, cl, _ = p.op
            n_loc = p.n_in + p.n_halo
            J = p.Jin[l]
            dZ = np.where(p.H[l] > 0, J, np.float32(0)).astype(np.float32) if l != L else J
            P = p.P[l - 1]
            a_dst, a_src = att[l - 1]
            dP = np.empty((n_loc, h), np.float32)
            da_dst = np.empty(h, np.float32)
            da_src = np.empty(h, np.float32)
            for k in range(heads):
                sl = slice(k * F, (k + 1) * F)
                Pk = np.ascontiguousarray(P[:, sl])
                dZk = np.ascontiguousarray(dZ[:, sl])
                alpha = p.alpha[l - 1][k]
                dalpha = O.sddmm(rp, cl, dZk, Pk, F)
                de = O.edge_softmax_bwd(rp, cl, alpha, dalpha, p.s_dst[l - 1][k], p.s_src[l - 1][k], slope)
                ds_dst = O.segment_sum(rp, de)
                ds_src = O.column_sum(rp, cl, n_loc, de)
                dPk = O.aggregate_bwd(rp, cl, alpha, n_loc, dZk, F)
                O.rank1_add(dPk, n_loc, ds_src, np.ascontiguousarray(a_src[sl]))
                O.rank1_add(dPk, p.n_in, ds_dst, np.ascontiguousarray(a_dst[sl]))
                dP[:, sl] = dPk
                da_dst[sl] = (Pk[: p.n_in].astype(np.float64).T @ ds_dst.astype(np.float64)).astype(np.float32)
                da_src[sl] = (Pk.astype(np.float64).T @ ds_src.astype(np.float64)).astype(np.float32)
            r = O.transform_bwd(p.Htil[l - 1], W[l - 1], False, dP, dP, want_dA=need_dx)
            p.G[l] = r["G"]
            p.Gatt[l] = (da_dst, da_src)
            dHt.append(r["dA1"] if need_dx else None)
        if need_dx:
            _exchange_rows_bwd(parts, dHt, l, seed, wire)
