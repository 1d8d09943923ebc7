"""The five synthetic workloads and the recipe that turns one into tensors.

Each workload takes the shape of one of the graphs the method was evaluated on
(node count, degree, feature width, model depth) and stands in for it; nothing
here is real data.  `scaled()` shrinks a workload for CPU-sized tests while
keeping its degree, widths and model.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List

import torch

from .graphs import er_edges, rmat_edges, partition_by_range, loopback_mirror, Partition


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    graph: str            # "er" | "rmat"
    n_nodes: int
    avg_deg: float
    n_parts: int          # node-range partitions; partition 0 is the one kept
    model: str            # "gcn" | "sage"
    dims: tuple           # (d_0, d_1, ..., d_L): layer l maps d_{l-1} -> d_l
    heavy_tail: bool      # per-row LogNormal(0, 2) scale on the input features
    seed: int
    all_parts: bool = False   # build every partition (real peers) instead of loopback


CONFIGS = {
    "tiny": WorkloadSpec("tiny", "er", 10_000, 10.0, 2, "gcn", (64, 64), False, 20230301 + 1,
                         all_parts=True),
    "dense_social": WorkloadSpec("dense_social", "rmat", 233_000, 490.0, 8, "gcn",
                                 (602, 256, 256), False, 20230301 + 2),
    "co_purchase": WorkloadSpec("co_purchase", "rmat", 2_450_000, 50.0, 8, "sage",
                                (100, 128, 128, 128), False, 20230301 + 3),
    "citation": WorkloadSpec("citation", "rmat", 2_900_000, 20.0, 8, "gcn",
                             (128, 256, 256, 256), False, 20230301 + 4),
    "stress": WorkloadSpec("stress", "rmat", 10_000_000, 32.0, 4, "gcn",
                           (256, 256, 256, 256, 256), True, 20230301 + 5),
}


def scaled(spec: WorkloadSpec, n_nodes: int, avg_deg: float | None = None) -> WorkloadSpec:
    """Same workload on fewer nodes (degree capped so the graph stays sparse)."""
    deg = spec.avg_deg if avg_deg is None else avg_deg
    deg = min(deg, n_nodes / 8)
    return replace(spec, name=f"{spec.name}@{n_nodes}", n_nodes=n_nodes, avg_deg=deg)


@dataclass
class Workload:
    spec: WorkloadSpec
    parts: List[Partition]        # partition 0 only, unless spec.all_parts
    mirror: torch.Tensor | None   # int32 [n_halo] loopback map (None with real peers)
    X: List[torch.Tensor]         # per partition: fp32 [n_in, d_0]
    W: List[torch.Tensor]         # per layer: fp32 [k_l, d_l], k_l = d_{l-1} (gcn) or 2 d_{l-1} (sage)
    J: List[torch.Tensor]         # per partition: upstream gradient fp32 [n_in, d_L]
    n_edges_undirected: int
    labels: List[torch.Tensor] = None   # per partition: int32 [n_in] class in [0, d_L), -1 = unlabelled


def build_workload(spec: WorkloadSpec, device="cpu") -> Workload:
    if spec.graph == "er":
        u, v = er_edges(spec.n_nodes, spec.avg_deg, spec.seed, device)
    elif spec.graph == "rmat":
        u, v = rmat_edges(spec.n_nodes, spec.avg_deg, spec.seed, device=device)
    else:
        raise ValueError(spec.graph)
    which = range(spec.n_parts) if spec.all_parts else range(1)
    parts = [partition_by_range(u, v, spec.n_nodes, spec.n_parts, p) for p in which]
    n_und = int(u.numel())
    del u, v
    g = torch.Generator(device=device)
    g.manual_seed(spec.seed * 7919 + 11)
    X, J = [], []
    for p in parts:
        x = torch.randn(p.n_in, spec.dims[0], generator=g, device=device, dtype=torch.float32)
        if spec.heavy_tail:
            f = torch.exp(2.0 * torch.randn(p.n_in, 1, generator=g, device=device,
                                            dtype=torch.float32))
            x = x * f
        X.append(x)
        J.append(torch.randn(p.n_in, spec.dims[-1], generator=g, device=device,
                             dtype=torch.float32) / p.n_in)
    W = []
    for l in range(1, len(spec.dims)):
        k = spec.dims[l - 1] * (2 if spec.model == "sage" else 1)
        W.append(torch.randn(k, spec.dims[l], generator=g, device=device,
                             dtype=torch.float32) / k ** 0.5)
    mirror = None
    if not spec.all_parts:
        mirror = loopback_mirror(parts[0].n_halo, parts[0].n_in, spec.seed + 77, device)
    # node labels for the training step: uniform classes, about 60 % of the nodes labelled
    # (own generator, so that everything above is unchanged by their presence)
    gl = torch.Generator(device=device)
    gl.manual_seed(spec.seed * 104729 + 5)
    labels = []
    for p in parts:
        y = torch.randint(0, spec.dims[-1], (p.n_in,), generator=gl, device=device, dtype=torch.int32)
        keep = torch.rand(p.n_in, generator=gl, device=device) < 0.6
        labels.append(torch.where(keep, y, torch.full_like(y, -1)))
    return Workload(spec, parts, mirror, X, W, J, n_und, labels)
