"""Seeded random graphs and node-range partitions.

Everything here is integer structure drawn with torch's seeded generators; it
runs unchanged on the CPU (small cases, CPU tests) and on a GPU (the large
workloads).  A graph is a set of undirected edges {u, v}, u != v, stored once
with u < v.  A partition keeps the rows of one contiguous node-id range and
names every neighbour outside that range a halo row.
"""
from __future__ import annotations

from dataclasses import dataclass
import math

import torch


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _unique_undirected(u: torch.Tensor, v: torch.Tensor, n_nodes: int):
    """Drop self loops and duplicate pairs; return sorted canonical keys lo*n+hi."""
    keep = u != v
    u, v = u[keep], v[keep]
    lo = torch.minimum(u, v)
    hi = torch.maximum(u, v)
    return torch.unique(lo * n_nodes + hi)


def er_edges(n_nodes: int, avg_deg: float, seed: int, device="cpu"):
    """Erdos-Renyi G(n, M) with M = n*avg_deg/2 distinct undirected edges."""
    g = _gen(seed, device)
    m = int(round(n_nodes * avg_deg / 2))
    keys = torch.empty(0, dtype=torch.int64, device=device)
    while keys.numel() < m:
        want = int((m - keys.numel()) * 1.1) + 16
        u = torch.randint(0, n_nodes, (want,), generator=g, device=device)
        v = torch.randint(0, n_nodes, (want,), generator=g, device=device)
        keys = torch.unique(torch.cat([keys, _unique_undirected(u, v, n_nodes)]))
    if keys.numel() > m:
        sel = torch.randperm(keys.numel(), generator=g, device=device)[:m]
        keys = keys[sel].sort().values
    return keys // n_nodes, keys % n_nodes


def rmat_edges(n_nodes: int, avg_deg: float, seed: int, a=0.57, b=0.19, c=0.19,
               device="cpu", chunk=1 << 24):
    """R-MAT (recursive quadrant) graph on n_nodes with about n*avg_deg/2 distinct edges.

    Ids are drawn on ceil(log2 n) bits, ids >= n_nodes are rejected, the ids are
    then relabelled by a random permutation (so a node-id range is a random node
    subset) and duplicate pairs and self loops are dropped.  Generation repeats
    until the distinct-edge target is reached, then a random subset of exactly
    that many edges is kept.
    """
    g = _gen(seed, device)
    bits = max(1, math.ceil(math.log2(n_nodes)))
    m = int(round(n_nodes * avg_deg / 2))
    perm = torch.randperm(n_nodes, generator=g, device=device)
    keys = torch.empty(0, dtype=torch.int64, device=device)
    ab, abc = a + b, a + b + c
    rounds = 0
    while keys.numel() < m:
        rounds += 1
        missing = m - keys.numel()
        # dense targets lose many draws to duplicates: oversample harder each round
        want = int(missing * (1.15 + 0.5 * (rounds - 1))) + 1024
        parts = [keys]
        for s in range(0, want, chunk):
            k = min(chunk, want - s)
            u = torch.zeros(k, dtype=torch.int64, device=device)
            v = torch.zeros(k, dtype=torch.int64, device=device)
            for _ in range(bits):
                r = torch.rand(k, generator=g, device=device)
                down = r >= ab                      # quadrants c, d: lower half of rows
                right = ((r >= a) & (r < ab)) | (r >= abc)   # quadrants b, d
                u = u * 2 + down.to(torch.int64)
                v = v * 2 + right.to(torch.int64)
            ok = (u < n_nodes) & (v < n_nodes)
            parts.append(_unique_undirected(perm[u[ok]], perm[v[ok]], n_nodes))
        keys = torch.unique(torch.cat(parts))
        if rounds > 64:
            raise RuntimeError("rmat_edges: distinct-edge target not reachable")
    if keys.numel() > m:
        sel = torch.randperm(keys.numel(), generator=g, device=device)[:m]
        keys = keys[sel].sort().values
    return keys // n_nodes, keys % n_nodes


@dataclass
class Partition:
    """One node-range partition of an undirected graph.

    Rows 0..n_in-1 are the inner nodes (global id lo + row); rows n_in..n_in+n_halo-1
    are the halo nodes in ascending global id.  (rowptr, col) is the adjacency of
    the inner rows over all n_in+n_halo local rows: no self loops, columns ascending
    within a row, no weights.  deg holds the global degree (distinct neighbours in
    the whole graph, self loop not counted) of every local row.  halo_part /
    halo_row name, for each halo row, the partition that owns the node and its row
    in that partition's inner block.
    """
    part: int
    lo: int
    n_in: int
    n_halo: int
    rowptr: torch.Tensor      # int64 [n_in+1]
    col: torch.Tensor         # int32 [nnz]
    deg: torch.Tensor         # int32 [n_in+n_halo]
    halo_gid: torch.Tensor    # int64 [n_halo]
    halo_part: torch.Tensor   # int32 [n_halo]
    halo_row: torch.Tensor    # int32 [n_halo]

    @property
    def nnz(self) -> int:
        return int(self.col.numel())


def partition_by_range(u: torch.Tensor, v: torch.Tensor, n_nodes: int, n_parts: int,
                       part: int) -> Partition:
    """Partition `part` of n_parts equal contiguous id ranges of the graph {u, v}."""
    width = -(-n_nodes // n_parts)
    lo = part * width
    hi = min(n_nodes, lo + width)
    n_in = hi - lo
    dev = u.device
    deg_all = torch.bincount(u, minlength=n_nodes) + torch.bincount(v, minlength=n_nodes)

    m1 = (u >= lo) & (u < hi)
    m2 = (v >= lo) & (v < hi)
    s = torch.cat([u[m1], v[m2]]) - lo          # local source row
    t = torch.cat([v[m1], u[m2]])               # global neighbour id
    outside = (t < lo) | (t >= hi)
    halo_gid = torch.unique(t[outside])
    n_halo = int(halo_gid.numel())
    col = torch.where(outside, n_in + torch.searchsorted(halo_gid, t), t - lo)
    # within a row: inner neighbours (ascending id) then halo neighbours (ascending id)
    order = torch.argsort(s * (n_in + n_halo) + col)
    s, col = s[order], col[order]
    rowptr = torch.zeros(n_in + 1, dtype=torch.int64, device=dev)
    rowptr[1:] = torch.cumsum(torch.bincount(s, minlength=n_in), 0)
    deg = torch.cat([deg_all[lo:hi], deg_all[halo_gid]]).to(torch.int32)
    return Partition(
        part=part, lo=lo, n_in=n_in, n_halo=n_halo, rowptr=rowptr,
        col=col.to(torch.int32), deg=deg, halo_gid=halo_gid,
        halo_part=(halo_gid // width).to(torch.int32),
        halo_row=(halo_gid % width).to(torch.int32),
    )


def loopback_mirror(n_halo: int, n_in: int, seed: int, device="cpu") -> torch.Tensor:
    """Stand-in for absent peers: halo row j is fed from inner row mirror[j].

    Drawn uniformly with replacement, so several halo rows share one inner row
    whenever n_halo is comparable to n_in (duplicates in the backward scatter).
    """
    g = _gen(seed, device)
    return torch.randint(0, n_in, (n_halo,), generator=g, device=device).to(torch.int32)
