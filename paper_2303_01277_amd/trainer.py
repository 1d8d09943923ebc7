"""Per-layer call sequence of Sylvie-S on one GPU (Alg. 1 forward, Alg. 2 backward), and
of Sylvie-A (Sec. 3.3): the same calls, but every layer computes with the wires received
in the previous epoch while this epoch's wires are produced on a second stream, with a
sequential epoch every eps_s epochs (Bounded Staleness Adaptor).

Every partition handed in lives on the same GPU; "send / receive" is the wire
arrays staying where the quantizer wrote them.  This module only allocates device
buffers and calls the C-ABI entry points in order: all arithmetic happens in the
HIP kernels.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, List, Optional

import contextlib

import torch

from . import binding as B
from . import graph_engine as GE


def default_pair_seed(seed: int, sender: int, receiver: int) -> int:
    return (int(seed) + 0x9E3779B97F4A7C15 * (sender * 4096 + receiver + 1)) & (2**64 - 1)


@dataclass
class Block:
    """Halo rows [j0, j1) of a receiver, all owned by partition `owner`."""
    owner: int
    j0: int
    j1: int
    rows: torch.Tensor          # int32 [j1-j0] owner-local inner rows (send list / scatter targets)
    seg_ptr: torch.Tensor
    seg_rows: torch.Tensor
    dst_ids: torch.Tensor
    planT: tuple = None         # long-row plan of the transposed operator on these halo rows
    orderT: Optional[torch.Tensor] = None   # processing order of these halo rows (longest first)
    inb_off: int = 0            # first row of this block in the owner's inbound wire


@dataclass
class PartState:
    n_in: int
    n_halo: int
    op: tuple                   # (rowptr, col, w) forward operator
    opT: tuple                  # transposed operator
    plan: tuple                 # long-row plan of op
    planT: tuple                # long-row plan of opT
    blocks: List[Block]
    X: torch.Tensor
    J: torch.Tensor
    Htil: List[torch.Tensor] = field(default_factory=list)   # Htil[l-1]: input of layer l
    Z: List[torch.Tensor] = field(default_factory=list)      # Z[l-1]: aggregate of layer l
    out: Optional[torch.Tensor] = None                        # H^(L)
    G: List[Optional[torch.Tensor]] = field(default_factory=list)
    dHtil: List[Optional[torch.Tensor]] = field(default_factory=list)  # dHtil[l-1]; J^(l-1) = its inner rows
    dZ: Optional[torch.Tensor] = None
    dself: Optional[torch.Tensor] = None
    ws_agg: Optional[torch.Tensor] = None
    ws_aggT: Optional[torch.Tensor] = None
    ws_g: Optional[torch.Tensor] = None
    wire: Optional[torch.Tensor] = None                       # int64 words, n_halo wire rows
    # fused backward: gradients arriving from every sender, concatenated (sender ascending)
    inbound: Optional[torch.Tensor] = None                    # int64 words, n_inbound wire rows
    n_inbound: int = 0
    inb_seg_ptr: Optional[torch.Tensor] = None                # int64 [n_in + 1]
    inb_seg_rows: Optional[torch.Tensor] = None               # int32 [n_inbound]
    planT_inner: tuple = None
    # processing orders (longest row first) of the operator's rows, of all rows of its transpose
    # and of the transpose's inner rows; None = index order
    order: Optional[torch.Tensor] = None
    orderT: Optional[torch.Tensor] = None
    orderT_inner: Optional[torch.Tensor] = None
    # pipeline mode: one wire per layer and two generations of each (this epoch / previous)
    fwd_wires: Optional[list] = None                          # [gen][l] int64 words
    inb_wires: Optional[list] = None                          # [gen][l] int64 words
    ws_aggT2: Optional[torch.Tensor] = None                   # long-row workspace of the side stream


WIRE_BITS = {"1bit": 1, "2bit": 2, "4bit": 4, "8bit": 8, "fp16": 16, "fp32": 32}


class LayerLoop:
    """model: "gcn" (A_hat = D^-1/2 (A+I) D^-1/2, H = sigma(A_hat Htil W)) or "sage"
    (mean aggregator, H = sigma([H_self | mean] W)).  ReLU on all layers but the last."""

    def __init__(self, parts, halo_owner, halo_row, X, J, W, model: str, dims, chunk: int = 1024,
                 exchange_first_layer: bool = False, wire: str = "1bit", fused: bool = True,
                 fused_bwd: bool = True, pipeline: bool = False, pad_wire: bool = True,
                 reorder: bool = False):
        """parts: synth Partition objects already on the GPU; halo_owner / halo_row: per
        partition int32 tensors naming the owner partition and owner-local inner row of
        each halo row (grouped by owner, ascending).  pad_wire: keep the resident 1-bit wire
        rows that the forward aggregation gathers at a line-friendly stride (see _stride)."""
        self.model, self.dims, self.W = model, tuple(dims), W
        self.L = len(W)
        self.chunk = chunk
        self.exchange_first_layer = exchange_first_layer
        self.wire = wire
        self.pad_wire = pad_wire
        # reorder: every aggregation launch hands its rows out longest first (same results bit
        # for bit).  Off by default: an L2 model predicts 11-15 % less traffic for it on the
        # stress partition, the chip's counters show none and the scattered row pointers cost
        # 5-28 % time; the hook stays for graphs whose own structure gives a better order.
        self.reorder = reorder
        if wire not in WIRE_BITS:
            raise ValueError(f"wire must be one of {sorted(WIRE_BITS)}")
        # bits per element on the wire: 1 = the paper's default; 2, 4, 8 and 16 (binary16)
        # are the other points of its bit-width study (Sec. 4.3); 32 = float rows, unchanged
        self.bits = WIRE_BITS.get(wire)
        # fused: the forward aggregation reads halo rows straight from the packed wire
        # (no dequantize pass, no float halo block)
        # (the wider codes of the bit-width study too, when every width is a multiple of 4)
        fusable = wire == "1bit" or (wire in ("2bit", "4bit", "8bit", "fp16") and all(d % 4 == 0 for d in dims))
        self.fused = fused and fusable
        # fused_bwd: the transposed aggregation quantizes the halo gradients on the spot
        # and adds the received ones in its epilogue (no float halo-gradient block, no
        # separate quantize / dequantize passes)
        self.fused_bwd = fused_bwd and fusable
        self.record = None          # set to a dict to keep copies of every wire
        self.part_streams = None    # one stream per partition while a step is being recorded (StepGraph)
        # pipeline: keep every layer's wires of this and of the previous epoch so that an
        # epoch can run on the previous epoch's wires (mode "async" of forward / backward)
        self.pipeline = pipeline
        if pipeline and wire != "1bit":
            raise ValueError("pipeline mode is built for the 1-bit wire")
        self.gen = 0                # generation that holds the wires of the running epoch
        self.have_prev = False
        dev = X[0].device
        self.dev = dev
        dmax = max(dims)
        self.parts: List[PartState] = []
        for p, part in enumerate(parts):
            if model == "gcn":
                op = GE.gcn_operator(part.rowptr, part.col, part.deg, part.n_in)
            else:
                op = GE.mean_operator(part.rowptr, part.col, part.n_in)
            n_loc = part.n_in + part.n_halo
            *opT, perm = GE.transpose_csr(op[0], op[1], op[2], n_loc, want_perm=True)
            opT = tuple(opT)
            plan = GE.long_row_plan(op[0], chunk)
            planT = GE.long_row_plan(opT[0], chunk)
            order = GE.rows_by_length(op[0]) if reorder else None
            orderT = GE.rows_by_length(opT[0]) if reorder else None
            blocks = []
            if part.n_halo:
                own, cnt = torch.unique_consecutive(halo_owner[p], return_counts=True)
                j = 0
                for o, c in zip(own.tolist(), cnt.tolist()):
                    rows = halo_row[p][j:j + c].contiguous()
                    sp, sr, di = GE.scatter_segments(rows, parts[o].n_in)
                    blocks.append(Block(o, j, j + c, rows, sp, sr, di))
                    j += c
            st = PartState(part.n_in, part.n_halo, op, opT, plan, planT, blocks, X[p], J[p])
            st.perm = perm              # entry i of opT is entry perm[i] of op
            st.order, st.orderT = order, orderT
            Wd = max(self._stride(d) for d in dims[:-1])
            st.wire = torch.empty(max(1, part.n_halo) * Wd, dtype=torch.int64, device=dev)
            st.ws_agg = torch.empty(max(1, plan[2]) * dmax, dtype=torch.float32, device=dev)
            st.ws_aggT = torch.empty(max(1, planT[2]) * dmax, dtype=torch.float32, device=dev)
            # per layer: the slab count, hence the size, depends on the layer's own widths
            nbytes = max(B.sylvie_transform_bwd_workspace_bytes(dims[l - 1] * (2 if model == "sage" else 1), 0,
                                                                dims[l], part.n_in)
                         for l in range(1, self.L + 1))
            st.ws_g = torch.empty(nbytes // 4, dtype=torch.float32, device=dev)
            for l in range(1, self.L + 1):
                # the float halo block below the inner rows exists only when it is written
                rows = part.n_in if self.fused else n_loc
                st.Htil.append(torch.empty(rows, dims[l - 1], dtype=torch.float32, device=dev))
                st.Z.append(torch.empty(part.n_in, dims[l - 1], dtype=torch.float32, device=dev))
            st.Htil[0][: part.n_in].copy_(X[p])
            st.out = torch.empty(part.n_in, dims[-1], dtype=torch.float32, device=dev)
            st.G = [None] + [torch.empty(W[l - 1].shape, dtype=torch.float32, device=dev)
                             for l in range(1, self.L + 1)]
            st.dHtil = [None] * self.L
            lo = 0 if exchange_first_layer else 1
            for l in range(lo, self.L):
                rows = part.n_in if self.fused_bwd else n_loc
                st.dHtil[l] = torch.empty(rows, dims[l], dtype=torch.float32, device=dev)
            st.dZ = torch.empty(part.n_in, dmax, dtype=torch.float32, device=dev)
            if model == "sage":
                st.dself = torch.empty(part.n_in, dmax, dtype=torch.float32, device=dev)
            self.parts.append(st)
        if self.fused_bwd or pipeline:
            Wd = self._words(dmax)
            for q, sq in enumerate(self.parts):
                dst = []
                for p, sp_ in enumerate(self.parts):
                    for b in sp_.blocks:
                        if b.owner != q:
                            continue
                        b.inb_off = sq.n_inbound
                        b.planT = GE.long_row_plan(sp_.opT[0], chunk, sp_.n_in + b.j0,
                                                   sp_.n_in + b.j1)
                        b.orderT = GE.rows_by_length(sp_.opT[0], sp_.n_in + b.j0,
                                                     sp_.n_in + b.j1) if reorder else None
                        sq.n_inbound += b.j1 - b.j0
                        dst.append(b.rows)
                dst = torch.cat(dst) if dst else torch.zeros(0, dtype=torch.int32, device=dev)
                sq.inb_seg_ptr, sq.inb_seg_rows = GE.scatter_segments_dense(dst, sq.n_in)
                sq.inbound = torch.empty(max(1, sq.n_inbound) * Wd, dtype=torch.int64, device=dev)
                sq.planT_inner = GE.long_row_plan(sq.opT[0], chunk, 0, sq.n_in)
                sq.orderT_inner = GE.rows_by_length(sq.opT[0], 0, sq.n_in) if reorder else None
        if pipeline:
            self.side = torch.cuda.Stream()        # default priority
            lo = 1 if exchange_first_layer else 2  # layers whose backward exchanges gradients
            for st in self.parts:
                st.fwd_wires = [[None] * (self.L + 1) for _ in range(2)]
                st.inb_wires = [[None] * (self.L + 1) for _ in range(2)]
                for g in range(2):
                    for l in range(1, self.L + 1):
                        Wl = B.sylvie_wire_row_words(dims[l - 1])
                        st.fwd_wires[g][l] = torch.empty(max(1, st.n_halo) * self._stride(dims[l - 1]),
                                                         dtype=torch.int64, device=dev)
                        if l >= lo:
                            st.inb_wires[g][l] = torch.empty(max(1, st.n_inbound) * Wl,
                                                             dtype=torch.int64, device=dev)
                st.ws_aggT2 = torch.empty_like(st.ws_aggT)

    # -- helpers ---------------------------------------------------------------
    def _keep(self, key, wire, n, W, stride=None):
        """Copy of n wire rows of W words each, packed, whatever stride they are kept at."""
        if self.record is not None:
            if stride is None or stride == W:
                self.record[key] = wire[: n * W].clone()
            else:
                self.record[key] = wire[: n * stride].view(n, stride)[:, :W].reshape(-1).clone()

    def _stride(self, d):
        """64-bit words between the resident wire rows that the forward aggregation gathers.
        A gathered 1-bit row costs one 128-byte line if it does not straddle one: the row's
        words are rounded up to a power of two (5 -> 8 words at d = 256), beyond 16 words to a
        multiple of 16.  The rows still travel packed: the padding is never written or read.
        Other wires (wider codes, gradient wires, which are read once in order) stay packed."""
        W = self._words(d)
        if self.bits != 1 or not self.pad_wire:
            return W
        if W > 16:
            return (W + 15) // 16 * 16
        S = 1
        while S < W:
            S *= 2
        return S

    def _words(self, d):
        """64-bit words of one wire row of width d."""
        if self.bits == 1:
            return B.sylvie_wire_row_words(d)
        return B.sylvie_wire_row_words_bits(d, self.bits)

    def _aggregate(self, fn, op, plan, ws, n_rows, X, d, Y, addend=None, addend_rows=0, order=None):
        rp, cl, w = op
        lr, lp, nt = plan
        fn(rp, cl, w, None, None, n_rows, X, X.stride(0), d, Y, Y.stride(0),
           addend=addend, ld_addend=0 if addend is None else addend.stride(0),
           addend_rows=addend_rows, chunk=self.chunk, long_rows=lr if nt else None,
           long_ptr=lp if nt else None, n_long=int(lr.numel()) if nt else 0, n_tasks=nt,
           workspace=ws if nt else None, row_order=order)

    def _each(self):
        """The partitions of one phase whose launches are independent of each other (each
        writes only its own buffers, or disjoint parts of a peer's).  Normally all on the
        caller's stream; with `part_streams` set (a step being recorded as a graph) partition p's
        launches go to stream p, forked from the caller's stream at the start of the phase and
        joined to it at the end, so that the recorded graph runs the partitions side by side."""
        streams = self.part_streams
        if not streams:
            yield from enumerate(self.parts)
            return
        cur = torch.cuda.current_stream()
        fork = torch.cuda.Event()
        fork.record(cur)
        for me, st in enumerate(self.parts):
            streams[me].wait_event(fork)
            with torch.cuda.stream(streams[me]):
                yield me, st
        for s in streams:
            cur.wait_stream(s)

    def _exchange_forward(self, l, d, Wd, seed, pair_seed):
        """Alg. 1, the exchange of layer l: every owner quantizes the rows its peers need; the
        receiver keeps the wire (fused aggregation) or recovers the rows into its halo block."""
        for me, st in self._each():
            ht = st.Htil[l - 1]
            for b in st.blocks:
                n = b.j1 - b.j0
                src = self.parts[b.owner].Htil[l - 1]
                if self.wire == "1bit":
                    # the wire of halo rows [j0, j1) sits at the same offset in the
                    # receiver's wire arrays, so all blocks stay resident side by side
                    S = self._stride(d)
                    wire = st.wire[b.j0 * S:]
                    B.sylvie_quantize_1bit_fwd(src, src.stride(0), d, b.rows, 0, n,
                                               pair_seed(seed, b.owner, me), 2 * l + 0, wire, ld_wire=S)
                    self._keep(("fwd", l, me, b.j0), wire, n, Wd, S)
                    if not self.fused:
                        B.sylvie_dequantize_1bit_fwd(wire, n, d, ht, ht.stride(0),
                                                     st.n_in + b.j0, ld_wire=S)
                else:   # wider codes, half precision, or the float rows themselves (bits = 32)
                    wire = st.wire[b.j0 * Wd:]
                    B.sylvie_quantize_bbit_fwd(src, src.stride(0), d, b.rows, 0, n, self.bits,
                                               pair_seed(seed, b.owner, me), 2 * l + 0, wire)
                    self._keep(("fwd", l, me, b.j0), wire, n, Wd)
                    if not self.fused:
                        B.sylvie_dequantize_bbit_fwd(wire, n, d, self.bits, ht, ht.stride(0),
                                                     st.n_in + b.j0)

    def _exchange_backward(self, l, d, Wd, seed, pair_seed):
        """Alg. 2, the exchange of layer l in two steps: quantize the halo block of every
        partition's gradient, add the recovered rows into the owners' inner rows."""
        # exchange the halo gradients; all transposed aggregates above are complete
        # before any partition's inner rows are touched (same stream, in order)
        for me, st in enumerate(self.parts):
            g = st.dHtil[l - 1]
            for b in st.blocks:
                n = b.j1 - b.j0
                tgt = self.parts[b.owner].dHtil[l - 1]
                if self.wire == "1bit":
                    B.sylvie_quantize_1bit_bwd(g, g.stride(0), d, None, st.n_in + b.j0, n,
                                               pair_seed(seed, me, b.owner), 2 * l + 1,
                                               st.wire)
                    self._keep(("bwd", l, me, b.j0), st.wire, n, Wd)
                    B.sylvie_dequantize_1bit_bwd(st.wire, n, d, tgt, tgt.stride(0), b.seg_ptr,
                                                 b.seg_rows, int(b.dst_ids.numel()), b.dst_ids)
                else:
                    B.sylvie_quantize_bbit_bwd(g, g.stride(0), d, None, st.n_in + b.j0, n,
                                               self.bits, pair_seed(seed, me, b.owner),
                                               2 * l + 1, st.wire)
                    self._keep(("bwd", l, me, b.j0), st.wire, n, Wd)
                    B.sylvie_dequantize_bbit_bwd(st.wire, n, d, self.bits, tgt, tgt.stride(0),
                                                 b.seg_ptr, b.seg_rows,
                                                 int(b.dst_ids.numel()), b.dst_ids)

    # -- Alg. 1 ------------------------------------------------------------------
    def forward(self, seed: int, pair_seed: Callable[[int, int, int], int] = default_pair_seed,
                mode: str = "sync"):
        if self.pipeline:
            return self._forward_pipeline(seed, pair_seed, mode)
        if mode != "sync":
            raise ValueError("mode 'async' needs pipeline=True")
        for l in range(1, self.L + 1):
            d = self.dims[l - 1]
            Wd = self._words(d)
            self._exchange_forward(l, d, Wd, seed, pair_seed)
            for _, st in self._each():
                ht, Z = st.Htil[l - 1], st.Z[l - 1]
                if self.fused:
                    rp, cl, w = st.op
                    lr, lp, nt = st.plan
                    B.sylvie_aggregate_csr_fwd_wire(
                        rp, cl, w, None, None, st.n_in, ht, ht.stride(0), d, st.n_in, st.wire,
                        st.n_halo, Z, Z.stride(0), chunk=self.chunk,
                        long_rows=lr if nt else None, long_ptr=lp if nt else None,
                        n_long=int(lr.numel()) if nt else 0, n_tasks=nt,
                        workspace=st.ws_agg if nt else None, ld_wire=self._stride(d),
                        row_order=st.order, bits=self.bits)
                else:
                    self._aggregate(B.sylvie_aggregate_csr_fwd, st.op, st.plan, st.ws_agg,
                                    st.n_in, ht, d, Z, order=st.order)
                relu = l != self.L
                Hout = st.Htil[l] if l < self.L else st.out
                h = self.dims[l]
                if self.model == "gcn":
                    B.sylvie_transform_fwd(Z, Z.stride(0), d, None, 0, 0, self.W[l - 1], h, st.n_in,
                                           relu, Hout, Hout.stride(0))
                else:
                    B.sylvie_transform_fwd(ht, ht.stride(0), d, Z, Z.stride(0), d, self.W[l - 1], h,
                                           st.n_in, relu, Hout, Hout.stride(0))

    # -- Alg. 2 ------------------------------------------------------------------
    def backward(self, seed: int, pair_seed: Callable[[int, int, int], int] = default_pair_seed,
                 mode: str = "sync"):
        if self.pipeline:
            return self._backward_pipeline(seed, pair_seed, mode)
        if mode != "sync":
            raise ValueError("mode 'async' needs pipeline=True")
        for l in range(self.L, 0, -1):
            d, h = self.dims[l - 1], self.dims[l]
            need_dx = l > 1 or self.exchange_first_layer
            Wd = self._words(d)
            for _, st in self._each():
                relu = l != self.L
                Hout = st.Htil[l] if l < self.L else st.out
                Jl = st.J if l == self.L else st.dHtil[l]
                ht, Z = st.Htil[l - 1], st.Z[l - 1]
                dZ = st.dZ.view(-1)[: st.n_in * d].view(st.n_in, d)
                if self.model == "gcn":
                    B.sylvie_transform_bwd(Z, Z.stride(0), d, None, 0, 0, self.W[l - 1], h, st.n_in,
                                           relu, Hout, Hout.stride(0), Jl, Jl.stride(0), st.G[l],
                                           dZ if need_dx else None, d, None, 0, st.ws_g)
                    dself = None
                else:
                    dself = st.dself.view(-1)[: st.n_in * d].view(st.n_in, d)
                    B.sylvie_transform_bwd(ht, ht.stride(0), d, Z, Z.stride(0), d, self.W[l - 1], h,
                                           st.n_in, relu, Hout, Hout.stride(0), Jl, Jl.stride(0),
                                           st.G[l], dself if need_dx else None, d,
                                           dZ if need_dx else None, d, st.ws_g)
                if need_dx and not self.fused_bwd:
                    g = st.dHtil[l - 1]
                    self._aggregate(B.sylvie_aggregate_csr_bwd, st.opT, st.planT, st.ws_aggT,
                                    st.n_in + st.n_halo, dZ, d, g, addend=dself,
                                    addend_rows=st.n_in, order=st.orderT)
            if not need_dx:
                continue
            if self.fused_bwd:
                self._backward_exchange_fused(l, d, Wd, seed, pair_seed)
                continue
            self._exchange_backward(l, d, Wd, seed, pair_seed)

    def _backward_exchange_fused(self, l, d, Wd, seed, pair_seed):
        """Halo gradients: aggregate + quantize straight into the owner's inbound wire;
        then inner gradients: aggregate + add the inbound wire rows, one store per row."""
        for me, st in self._each():
            rpT, clT, wT = st.opT
            dZ = st.dZ.view(-1)[: st.n_in * d].view(st.n_in, d)
            for b in st.blocks:
                tgt = self.parts[b.owner]
                wire = tgt.inbound[b.inb_off * Wd:]
                lr, lp, nt = b.planT
                B.sylvie_aggregate_csr_bwd_quantize(
                    rpT, clT, wT, None, None, st.n_in + b.j0, b.j1 - b.j0, dZ, d, d,
                    pair_seed(seed, me, b.owner), 2 * l + 1, wire, chunk=self.chunk,
                    long_rows=lr if nt else None, long_ptr=lp if nt else None,
                    n_long=int(lr.numel()) if nt else 0, n_tasks=nt,
                    workspace=st.ws_aggT if nt else None, row_order=b.orderT, bits=self.bits)
                self._keep(("bwd", l, me, b.j0), wire, b.j1 - b.j0, Wd)
        for _, st in self._each():
            rpT, clT, wT = st.opT
            dZ = st.dZ.view(-1)[: st.n_in * d].view(st.n_in, d)
            dself = None
            if self.model == "sage":
                dself = st.dself.view(-1)[: st.n_in * d].view(st.n_in, d)
            g = st.dHtil[l - 1]
            lr, lp, nt = st.planT_inner
            B.sylvie_aggregate_csr_bwd_integrate(
                rpT, clT, wT, None, None, 0, st.n_in, dZ, d, d, g, g.stride(0), dself,
                0 if dself is None else d, st.n_in, st.inbound, st.n_inbound, st.inb_seg_ptr,
                st.inb_seg_rows, chunk=self.chunk, long_rows=lr if nt else None,
                long_ptr=lp if nt else None, n_long=int(lr.numel()) if nt else 0, n_tasks=nt,
                workspace=st.ws_aggT if nt else None, row_order=st.orderT_inner, bits=self.bits)

    # -- Sylvie-A (Sec. 3.3): pipeline mode ------------------------------------------
    def _gen(self, which):
        return self.gen if which == "cur" else self.gen ^ 1

    def _side(self, stale):
        """Context in which this epoch's wires are produced: the side stream when the layer
        computes with the previous epoch's wires, the caller's stream otherwise."""
        if not stale:
            return contextlib.nullcontext()
        self.side.wait_stream(torch.cuda.current_stream())
        return torch.cuda.stream(self.side)

    def _check_mode(self, mode):
        if mode not in ("sync", "async"):
            raise ValueError("mode must be 'sync' or 'async'")
        if mode == "async" and not self.have_prev:
            raise ValueError("the first epoch has no previous wires: run it with mode='sync'")
        return mode == "async"

    def _forward_pipeline(self, seed, pair_seed, mode):
        stale = self._check_mode(mode)
        main = torch.cuda.current_stream()
        use = "prev" if stale else "cur"
        for l in range(1, self.L + 1):
            d = self.dims[l - 1]
            Wd = B.sylvie_wire_row_words(d)
            S = self._stride(d)
            # this epoch's wires (every partition's H^(l-1) is complete on the main stream)
            with self._side(stale):
                for me, st in enumerate(self.parts):
                    cur = st.fwd_wires[self._gen("cur")][l]
                    for b in st.blocks:
                        src = self.parts[b.owner].Htil[l - 1]
                        wire = cur[b.j0 * S:]
                        B.sylvie_quantize_1bit_fwd(src, src.stride(0), d, b.rows, 0, b.j1 - b.j0,
                                                   pair_seed(seed, b.owner, me), 2 * l + 0, wire, ld_wire=S)
                        self._keep(("fwd", l, me, b.j0), wire, b.j1 - b.j0, Wd, S)
            for st in self.parts:
                ht, Z = st.Htil[l - 1], st.Z[l - 1]
                wire = st.fwd_wires[self._gen(use)][l]
                if self.fused:
                    rp, cl, w = st.op
                    lr, lp, nt = st.plan
                    B.sylvie_aggregate_csr_fwd_wire(
                        rp, cl, w, None, None, st.n_in, ht, ht.stride(0), d, st.n_in, wire,
                        st.n_halo, Z, Z.stride(0), chunk=self.chunk,
                        long_rows=lr if nt else None, long_ptr=lp if nt else None,
                        n_long=int(lr.numel()) if nt else 0, n_tasks=nt,
                        workspace=st.ws_agg if nt else None, ld_wire=S, row_order=st.order)
                else:
                    if st.n_halo:
                        B.sylvie_dequantize_1bit_fwd(wire, st.n_halo, d, ht, ht.stride(0), st.n_in,
                                                     ld_wire=S)
                    self._aggregate(B.sylvie_aggregate_csr_fwd, st.op, st.plan, st.ws_agg,
                                    st.n_in, ht, d, Z, order=st.order)
                relu = l != self.L
                Hout = st.Htil[l] if l < self.L else st.out
                h = self.dims[l]
                if self.model == "gcn":
                    B.sylvie_transform_fwd(Z, Z.stride(0), d, None, 0, 0, self.W[l - 1], h, st.n_in,
                                           relu, Hout, Hout.stride(0))
                else:
                    B.sylvie_transform_fwd(ht, ht.stride(0), d, Z, Z.stride(0), d, self.W[l - 1], h,
                                           st.n_in, relu, Hout, Hout.stride(0))
        if stale:
            main.wait_stream(self.side)

    def _backward_pipeline(self, seed, pair_seed, mode):
        stale = self._check_mode(mode)
        main = torch.cuda.current_stream()
        use = "prev" if stale else "cur"
        for l in range(self.L, 0, -1):
            d, h = self.dims[l - 1], self.dims[l]
            need_dx = l > 1 or self.exchange_first_layer
            Wd = B.sylvie_wire_row_words(d)
            for st in self.parts:
                relu = l != self.L
                Hout = st.Htil[l] if l < self.L else st.out
                Jl = st.J if l == self.L else st.dHtil[l]
                ht, Z = st.Htil[l - 1], st.Z[l - 1]
                dZ = st.dZ.view(-1)[: st.n_in * d].view(st.n_in, d)
                if self.model == "gcn":
                    B.sylvie_transform_bwd(Z, Z.stride(0), d, None, 0, 0, self.W[l - 1], h, st.n_in,
                                           relu, Hout, Hout.stride(0), Jl, Jl.stride(0), st.G[l],
                                           dZ if need_dx else None, d, None, 0, st.ws_g)
                    dself = None
                else:
                    dself = st.dself.view(-1)[: st.n_in * d].view(st.n_in, d)
                    B.sylvie_transform_bwd(ht, ht.stride(0), d, Z, Z.stride(0), d, self.W[l - 1], h,
                                           st.n_in, relu, Hout, Hout.stride(0), Jl, Jl.stride(0),
                                           st.G[l], dself if need_dx else None, d,
                                           dZ if need_dx else None, d, st.ws_g)
                if need_dx and not self.fused_bwd:
                    g = st.dHtil[l - 1]
                    self._aggregate(B.sylvie_aggregate_csr_bwd, st.opT, st.planT, st.ws_aggT,
                                    st.n_in + st.n_halo, dZ, d, g, addend=dself,
                                    addend_rows=st.n_in, order=st.orderT)
            if not need_dx:
                continue
            # this epoch's gradient wires, written into the owners' inbound buffers
            with self._side(stale):
                for me, st in enumerate(self.parts):
                    rpT, clT, wT = st.opT
                    dZ = st.dZ.view(-1)[: st.n_in * d].view(st.n_in, d)
                    g = st.dHtil[l - 1]
                    for b in st.blocks:
                        tgt = self.parts[b.owner]
                        wire = tgt.inb_wires[self._gen("cur")][l][b.inb_off * Wd:]
                        if self.fused_bwd:
                            lr, lp, nt = b.planT
                            ws = st.ws_aggT2 if stale else st.ws_aggT
                            B.sylvie_aggregate_csr_bwd_quantize(
                                rpT, clT, wT, None, None, st.n_in + b.j0, b.j1 - b.j0, dZ, d, d,
                                pair_seed(seed, me, b.owner), 2 * l + 1, wire, chunk=self.chunk,
                                long_rows=lr if nt else None, long_ptr=lp if nt else None,
                                n_long=int(lr.numel()) if nt else 0, n_tasks=nt,
                                workspace=ws if nt else None, row_order=b.orderT)
                        else:
                            B.sylvie_quantize_1bit_bwd(g, g.stride(0), d, None, st.n_in + b.j0,
                                                       b.j1 - b.j0, pair_seed(seed, me, b.owner),
                                                       2 * l + 1, wire)
                        self._keep(("bwd", l, me, b.j0), wire, b.j1 - b.j0, Wd)
            # integrate the gradient wires in use (Alg. 2, J = J + R~)
            for st in self.parts:
                inb = st.inb_wires[self._gen(use)][l]
                g = st.dHtil[l - 1]
                if self.fused_bwd:
                    rpT, clT, wT = st.opT
                    dZ = st.dZ.view(-1)[: st.n_in * d].view(st.n_in, d)
                    dself = None
                    if self.model == "sage":
                        dself = st.dself.view(-1)[: st.n_in * d].view(st.n_in, d)
                    lr, lp, nt = st.planT_inner
                    B.sylvie_aggregate_csr_bwd_integrate(
                        rpT, clT, wT, None, None, 0, st.n_in, dZ, d, d, g, g.stride(0), dself,
                        0 if dself is None else d, st.n_in, inb, st.n_inbound, st.inb_seg_ptr,
                        st.inb_seg_rows, chunk=self.chunk, long_rows=lr if nt else None,
                        long_ptr=lp if nt else None, n_long=int(lr.numel()) if nt else 0,
                        n_tasks=nt, workspace=st.ws_aggT if nt else None,
                        row_order=st.orderT_inner)
            if not self.fused_bwd:
                for sp_ in self.parts:
                    for b in sp_.blocks:
                        tgt = self.parts[b.owner]
                        inb = tgt.inb_wires[self._gen(use)][l][b.inb_off * Wd:]
                        gt = tgt.dHtil[l - 1]
                        B.sylvie_dequantize_1bit_bwd(inb, b.j1 - b.j0, d, gt, gt.stride(0),
                                                     b.seg_ptr, b.seg_rows, int(b.dst_ids.numel()),
                                                     b.dst_ids)
            if stale:
                main.wait_stream(self.side)    # dZ and the float halo block are reused next layer

    def step(self, seed: int, pair_seed: Callable[[int, int, int], int] = default_pair_seed,
             mode: str = "sync"):
        """One epoch (forward + backward); in pipeline mode its wires then become the
        previous epoch's."""
        self.forward(seed, pair_seed, mode)
        self.backward(seed, pair_seed, mode)
        if self.pipeline:
            self.gen ^= 1
            self.have_prev = True

    def run_epochs(self, n: int, seed0: int, eps_s: int = 0,
                   pair_seed: Callable[[int, int, int], int] = default_pair_seed):
        """Bounded Staleness Adaptor (Sec. 3.3): epoch e runs sequentially ("sync") when
        e == 0 or eps_s > 0 and e % eps_s == 0, in pipeline mode ("async") otherwise.
        Returns the list of modes."""
        modes = []
        for e in range(n):
            mode = "sync" if (e == 0 or not self.pipeline or (eps_s > 0 and e % eps_s == 0)) else "async"
            self.step(seed0 + e, pair_seed, mode)
            modes.append(mode)
        return modes

    # -- the rest of the training step (Alg. 1 last line, Alg. 2 first and last lines) -------
    def loss_and_gradient(self, labels, count: float):
        """J^(L) of every partition = gradient of the softmax cross-entropy of its H^(L) over its
        labelled nodes (labels[p] int32 [n_in], -1 = unlabelled; count = labelled nodes of the
        whole graph).  Returns the per-partition loss sums as a float64 GPU tensor."""
        if not hasattr(self, "_loss_rows"):
            self._loss_rows = [torch.empty(max(1, st.n_in), dtype=torch.float32, device=self.dev)
                               for st in self.parts]
            self._loss = torch.zeros(len(self.parts), dtype=torch.float64, device=self.dev)
        C_ = self.dims[-1]
        for p, st in enumerate(self.parts):
            B.sylvie_softmax_xent(st.out, st.out.stride(0), st.n_in, C_, labels[p], count, st.J,
                                  st.J.stride(0), self._loss_rows[p], self._loss[p:p + 1])
        return self._loss

    def update_weights(self, eta: float):
        """G = sum of the partitions' weight gradients (ascending partition order, the stand-in
        for the all-reduce between GPUs); W = W - eta G."""
        if not hasattr(self, "_gsum"):
            self._gsum = [None] + [torch.empty_like(w) for w in self.W]
        for l in range(1, self.L + 1):
            srcs = [st.G[l] for st in self.parts]
            B.sylvie_sum_gradients(self._gsum[l], srcs, len(srcs), self._gsum[l].numel())
            B.sylvie_sgd_update(self.W[l - 1], self._gsum[l], self.W[l - 1].numel(), eta)

    def train_step(self, seed: int, labels, count: float, eta: float,
                   pair_seed: Callable[[int, int, int], int] = default_pair_seed,
                   mode: str = "sync"):
        """forward -> loss and J^(L) -> backward -> gradient sum -> SGD update."""
        self.forward(seed, pair_seed, mode)
        loss = self.loss_and_gradient(labels, count)
        self.backward(seed, pair_seed, mode)
        if self.pipeline:
            self.gen ^= 1
            self.have_prev = True
        self.update_weights(eta)
        return loss


class StepGraph:
    """One epoch of a layer loop (forward + backward, sequential mode) recorded once as a HIP
    graph and replayed: for small partitions the step is bound by its launches, not its kernels.
    The quantizing calls take their seed by value, so the graph is recorded with the library's
    device-resident seed offset switched on and ends with a kernel that advances it: replay k
    (k = 0, 1, ...) is the step with pair seeds pair_seed(seed, a, b) + k, bit for bit."""

    def __init__(self, loop: "LayerLoop", seed: int,
                 pair_seed: Callable[[int, int, int], int] = default_pair_seed):
        if loop.pipeline:
            raise ValueError("a recorded step runs in sequential mode")
        self.loop = loop
        self.epoch = torch.zeros(1, dtype=torch.int64, device=loop.dev)
        cur = torch.cuda.current_stream()
        side = torch.cuda.Stream()
        B.sylvie_seed_offset_source(self.epoch)
        if len(loop.parts) > 1 and not isinstance(loop, AttentionLoop):
            loop.part_streams = [torch.cuda.Stream() for _ in loop.parts]
        try:
            # one eager step on a side stream first, as the tensor library asks before a capture
            side.wait_stream(cur)
            with torch.cuda.stream(side):
                loop.step(seed, pair_seed)
            cur.wait_stream(side)
            torch.cuda.synchronize()
            self.graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(self.graph):
                loop.step(seed, pair_seed)
                self.epoch.add_(1)          # an ordinary kernel: no memset node in the graph
        finally:
            B.sylvie_seed_offset_source(None)
            loop.part_streams = None

    def replay(self):
        self.graph.replay()

    def reset(self, k: int = 0):
        """The next replay is replay number k."""
        self.epoch.fill_(k)


class AttentionLoop(LayerLoop):
    """The attention model (GAT) under the same exchange: layer l transforms inner and recovered
    halo rows, P = Htilde W, scores every operator entry with leaky_relu(P_v . a_dst + P_u . a_src),
    normalises the scores of each row with a softmax and aggregates Z = sum alpha P_u;
    H = relu(Z) except on the last layer.  `heads` attention heads share W column-wise: head k
    owns columns [k F, (k+1) F) of P, F = d_l / heads, and its own slices of a_dst / a_src.
    All heads go through one call per step: scores and per-entry values are [.][heads] arrays.
    The exchange is the two-step one (the transform needs the halo rows as floats)."""

    def __init__(self, parts, halo_owner, halo_row, X, J, W, att, dims, heads: int = 1,
                 slope: float = 0.2, chunk: int = 1024, exchange_first_layer: bool = False,
                 wire: str = "1bit", fused_sddmm: bool = True):
        super().__init__(parts, halo_owner, halo_row, X, J, W, "gcn", dims, chunk=chunk,
                         exchange_first_layer=exchange_first_layer, wire=wire, fused=False,
                         fused_bwd=False)
        self.model = "gat"
        self.att, self.heads, self.slope = att, heads, slope
        # layers whose transposed aggregation also forms the sampled product dalpha = dZ_v . P_u
        self.fused_sddmm = [False] + [fused_sddmm and B.sylvie_aggregate_csr_attention_sddmm_supported(dims[l], heads)
                                      and max(dims[1:]) % 4 == 0 for l in range(1, len(dims))]
        if heads not in (1, 2, 4, 8):
            raise ValueError("heads must be 1, 2, 4 or 8")
        if any(d % heads for d in dims[1:]):
            raise ValueError("every layer width must be a multiple of heads")
        dev = self.dev
        K = heads
        for st in self.parts:
            n_loc = st.n_in + st.n_halo
            nnz = int(st.op[0][-1])
            st.pieces = GE.piece_table(st.op[0], chunk)
            st.piecesT = GE.piece_table(st.opT[0], chunk)
            st.P = [None] + [torch.empty(n_loc, dims[l], dtype=torch.float32, device=dev)
                             for l in range(1, self.L + 1)]
            st.alpha = [None] + [torch.empty(nnz * K, dtype=torch.float32, device=dev) for _ in range(self.L)]
            st.s_dst = [None] + [torch.empty(st.n_in * K, dtype=torch.float32, device=dev) for _ in range(self.L)]
            st.s_src = [None] + [torch.empty(n_loc * K, dtype=torch.float32, device=dev) for _ in range(self.L)]
            st.edge = [torch.empty(nnz * K, dtype=torch.float32, device=dev) for _ in range(2)]
            st.ds_dst = torch.empty(st.n_in * K, dtype=torch.float32, device=dev)
            st.ds_src = torch.empty(n_loc * K, dtype=torch.float32, device=dev)
            st.dP = torch.empty(n_loc, max(dims[1:]), dtype=torch.float32, device=dev)
            st.dZg = torch.empty(st.n_in, max(dims[1:]), dtype=torch.float32, device=dev)
            n_ws = max(B.sylvie_edge_softmax_heads_workspace_bytes(st.pieces[1].numel(), st.n_in, K) // 4,
                       (st.piecesT[1].numel() + n_loc) * K, 1)
            st.ws_att = torch.empty(n_ws, dtype=torch.float32, device=dev)
            nbytes = max(B.sylvie_transform_bwd_workspace_bytes(dims[l - 1], 0, dims[l], n_loc)
                         for l in range(1, self.L + 1))
            st.ws_g = torch.empty(nbytes // 4, dtype=torch.float32, device=dev)
            st.Ga = [None] + [(torch.empty(dims[l], dtype=torch.float32, device=dev),
                               torch.empty(dims[l], dtype=torch.float32, device=dev))
                              for l in range(1, self.L + 1)]
            st.ws_col = torch.empty(max(1, 2 * B.sylvie_scaled_column_sum_workspace_bytes(n_loc, max(dims[1:])) // 4),
                                    dtype=torch.float32, device=dev)

    def forward(self, seed, pair_seed=default_pair_seed, mode="sync"):
        if mode != "sync":
            raise ValueError("the attention loop runs sequentially")
        K = self.heads
        for l in range(1, self.L + 1):
            d, h = self.dims[l - 1], self.dims[l]
            F = h // K
            self._exchange_forward(l, d, self._words(d), seed, pair_seed)
            a_dst, a_src = self.att[l - 1]
            for st in self.parts:
                n_loc = st.n_in + st.n_halo
                ht, P = st.Htil[l - 1], st.P[l]
                # the hidden layers' activation is the aggregation's last step
                Y = st.Htil[l] if l < self.L else st.out
                B.sylvie_transform_fwd(ht, ht.stride(0), d, None, 0, 0, self.W[l - 1], h, n_loc, False,
                                       P, P.stride(0))
                rp, cl, _ = st.op
                lr, lp, nt = st.plan
                sd, ss, al = st.s_dst[l], st.s_src[l], st.alpha[l]
                B.sylvie_row_dot_heads(P, h, st.n_in, F, K, a_dst, sd, a2=a_src, n2=n_loc, out2=ss)
                B.sylvie_edge_softmax_fwd_heads(st.pieces, cl, sd, ss, K, self.slope, al, st.ws_att)
                B.sylvie_aggregate_csr_attention(rp, cl, al, None, K, st.n_in, P, h, h, Y, Y.stride(0),
                                                 relu=l != self.L, chunk=self.chunk,
                                                 long_rows=lr if nt else None, long_ptr=lp if nt else None,
                                                 n_long=int(lr.numel()) if nt else 0, n_tasks=nt,
                                                 workspace=st.ws_agg if nt else None)

    def backward(self, seed, pair_seed=default_pair_seed, mode="sync"):
        if mode != "sync":
            raise ValueError("the attention loop runs sequentially")
        K = self.heads
        for l in range(self.L, 0, -1):
            d, h = self.dims[l - 1], self.dims[l]
            F = h // K
            need_dx = l > 1 or self.exchange_first_layer
            a_dst, a_src = self.att[l - 1]
            for st in self.parts:
                n_loc = st.n_in + st.n_halo
                Hout = st.Htil[l] if l < self.L else st.out
                Jl = st.J if l == self.L else st.dHtil[l]
                P, dP = st.P[l], st.dP
                if l != self.L:
                    dZ = st.dZg
                    B.sylvie_relu_bwd(Hout, Hout.stride(0), Jl, Jl.stride(0), st.n_in, h, dZ, dZ.stride(0))
                else:
                    dZ = Jl
                ldz, ldp = dZ.stride(0), dP.stride(0)
                _, cl, _ = st.op
                rpT, clT, _ = st.opT
                lr, lp, nt = st.planT
                dal, de = st.edge
                da_dst, da_src = st.Ga[l]
                sd, ss, al = st.s_dst[l], st.s_src[l], st.alpha[l]
                planT = dict(chunk=self.chunk, long_rows=lr if nt else None, long_ptr=lp if nt else None,
                             n_long=int(lr.numel()) if nt else 0, n_tasks=nt,
                             workspace=st.ws_aggT if nt else None)
                # column sums of de and the transposed aggregation read de / alpha in forward
                # entry order through the transposition's entry map
                if self.fused_sddmm[l]:
                    # the transposed aggregation gathers dZ_v per entry anyway: it also forms dalpha
                    B.sylvie_aggregate_csr_attention_sddmm(rpT, clT, al, st.perm, K, n_loc, dZ, ldz, h, dP, ldp,
                                                           P, h, dal, **planT)
                    B.sylvie_edge_softmax_bwd_heads(st.pieces, cl, al, dal, sd, ss, K, self.slope, de,
                                                    st.ds_dst, st.ws_att)
                    B.sylvie_segment_sum_heads(st.piecesT, de, st.perm, K, st.ds_src, st.ws_att)
                    B.sylvie_rank1_add_heads(dP, ldp, h, K, st.ds_src, a_src, n_loc, st.ds_dst, a_dst, st.n_in)
                else:
                    B.sylvie_sddmm_heads(st.pieces, cl, dZ, ldz, P, h, F, K, dal)
                    B.sylvie_edge_softmax_bwd_heads(st.pieces, cl, al, dal, sd, ss, K, self.slope, de,
                                                    st.ds_dst, st.ws_att)
                    B.sylvie_segment_sum_heads(st.piecesT, de, st.perm, K, st.ds_src, st.ws_att)
                    B.sylvie_aggregate_csr_attention(rpT, clT, al, st.perm, K, n_loc, dZ, ldz, h, dP, ldp,
                                                     s1=st.ds_src, a1=a_src, n1=n_loc,
                                                     s2=st.ds_dst, a2=a_dst, n2=st.n_in, **planT)
                B.sylvie_scaled_column_sum_heads(P, h, st.n_in, h, K, st.ds_dst, da_dst, st.ws_col,
                                                 s2=st.ds_src, n2=n_loc, out2=da_src)
                ht = st.Htil[l - 1]
                g = st.dHtil[l - 1] if need_dx else None
                B.sylvie_transform_bwd(ht, ht.stride(0), d, None, 0, 0, self.W[l - 1], h, n_loc, False,
                                       None, 0, dP, ldp, st.G[l], g, 0 if g is None else g.stride(0),
                                       None, 0, st.ws_g)
            if need_dx:
                self._exchange_backward(l, d, self._words(d), seed, pair_seed)

    def update_weights(self, eta: float):
        super().update_weights(eta)
        if not hasattr(self, "_gasum"):
            self._gasum = [None] + [(torch.empty_like(a), torch.empty_like(b)) for a, b in self.att]
        for l in range(1, self.L + 1):
            for i in (0, 1):
                srcs = [st.Ga[l][i] for st in self.parts]
                B.sylvie_sum_gradients(self._gasum[l][i], srcs, len(srcs), srcs[0].numel())
                B.sylvie_sgd_update(self.att[l - 1][i], self._gasum[l][i], srcs[0].numel(), eta)
