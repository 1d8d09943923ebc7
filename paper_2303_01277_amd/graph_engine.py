"""One-off set-up of a partition (the "Graph Engine" step, Sec. 3.2; Alg. 1 lines 3-7).

Builds, once per graph, the index structures the kernels consume: the normalised
operator of the partition (Sec. 3.4), its transpose as a CSR of its own, the plan
that cuts long rows into tasks, and the scatter segments of the backward
dequantizer.  All functions take and return torch tensors and run on whatever
device the inputs live on; none of this is on the per-layer hot path.
"""
from __future__ import annotations

import torch


def gcn_operator(rowptr, col, deg, n_in):
    """Rows of D^-1/2 (A + I) D^-1/2 for the inner nodes of a partition.

    rowptr/col: adjacency of the inner rows over all local rows (inner + halo), no
    self loops, columns ascending.  deg[r]: degree of local row r in the whole
    graph, self loop not counted.  Returns (rowptr', col', w) with the self loop
    (r, r) merged in column order and w = 1/sqrt((deg_r + 1)(deg_c + 1)) evaluated
    in float64, rounded once to float32.
    """
    dev = rowptr.device
    counts = rowptr[1:] - rowptr[:-1]
    rows = torch.repeat_interleave(torch.arange(n_in, device=dev), counts)
    self_rows = torch.arange(n_in, device=dev)
    all_rows = torch.cat([rows, self_rows])
    all_cols = torch.cat([col.to(torch.int64), self_rows])
    n_cols = int(deg.numel())
    order = torch.argsort(all_rows * n_cols + all_cols)
    all_rows, all_cols = all_rows[order], all_cols[order]
    new_rowptr = rowptr + torch.arange(n_in + 1, device=dev, dtype=torch.int64)
    d1 = deg.to(torch.float64) + 1.0
    w = (1.0 / torch.sqrt(d1[all_rows] * d1[all_cols])).to(torch.float32)
    return new_rowptr, all_cols.to(torch.int32), w


def mean_operator(rowptr, col, n_in):
    """GraphSAGE mean aggregator: every entry of row r weighs 1/len(r)."""
    counts = rowptr[1:] - rowptr[:-1]
    inv = (1.0 / counts.to(torch.float64)).to(torch.float32)
    w = torch.repeat_interleave(inv, counts)
    return rowptr, col, w


def transpose_csr(rowptr, col, w, n_cols):
    """CSR of the transposed operator: n_cols rows; entries of a row in ascending
    original-row order.  Returns (rowptrT int64, colT int32, wT float32)."""
    dev = rowptr.device
    n_rows = int(rowptr.numel()) - 1
    counts = rowptr[1:] - rowptr[:-1]
    rows = torch.repeat_interleave(torch.arange(n_rows, device=dev), counts)
    c64 = col.to(torch.int64)
    order = torch.argsort(c64 * n_rows + rows)
    rowptrT = torch.zeros(n_cols + 1, dtype=torch.int64, device=dev)
    rowptrT[1:] = torch.cumsum(torch.bincount(c64, minlength=n_cols), 0)
    return rowptrT, rows[order].to(torch.int32), w[order].contiguous()


def long_row_plan(rowptr, chunk, row_begin=0, row_end=None):
    """Rows longer than `chunk` entries (absolute indices, optionally only those in
    [row_begin, row_end)) and the prefix sum of their task counts.
    Returns (long_rows int32 [n_long], long_ptr int64 [n_long + 1], n_tasks)."""
    if chunk <= 0 or chunk % 64:
        raise ValueError("chunk must be a positive multiple of 64")
    counts = rowptr[1:] - rowptr[:-1]
    long_rows = torch.nonzero(counts > chunk).flatten()
    if row_end is not None or row_begin:
        hi = counts.numel() if row_end is None else row_end
        long_rows = long_rows[(long_rows >= row_begin) & (long_rows < hi)]
    tasks = (counts[long_rows] + chunk - 1) // chunk
    long_ptr = torch.zeros(long_rows.numel() + 1, dtype=torch.int64, device=rowptr.device)
    long_ptr[1:] = torch.cumsum(tasks, 0)
    return long_rows.to(torch.int32), long_ptr, int(long_ptr[-1])


def scatter_segments(dst_row):
    """Group wire rows by destination row for the backward dequantizer.

    dst_row int32 [n]: destination of wire row i.  Returns (seg_ptr int64 [m + 1],
    seg_rows int32 [n], dst_ids int32 [m]): destination dst_ids[k] receives wire
    rows seg_rows[seg_ptr[k] : seg_ptr[k+1]], ascending.
    """
    d64 = dst_row.to(torch.int64)
    order = torch.sort(d64, stable=True).indices
    dst_ids, counts = torch.unique_consecutive(d64[order], return_counts=True)
    seg_ptr = torch.zeros(dst_ids.numel() + 1, dtype=torch.int64, device=dst_row.device)
    seg_ptr[1:] = torch.cumsum(counts, 0)
    return seg_ptr, order.to(torch.int32), dst_ids.to(torch.int32)


def scatter_segments_dense(dst_row, n_dst):
    """Like scatter_segments, but with one (possibly empty) segment for every
    destination row 0 .. n_dst - 1: returns (seg_ptr int64 [n_dst + 1], seg_rows int32 [n])."""
    d64 = dst_row.to(torch.int64)
    order = torch.sort(d64, stable=True).indices
    seg_ptr = torch.zeros(n_dst + 1, dtype=torch.int64, device=dst_row.device)
    seg_ptr[1:] = torch.cumsum(torch.bincount(d64, minlength=n_dst), 0)
    return seg_ptr, order.to(torch.int32)


def piece_table(rowptr, chunk):
    """Cuts every row's entries into pieces of at most `chunk` consecutive entries (rows without
    entries get none).  Returns (piece_ptr int64 [n_pieces + 1], piece_row int32 [n_pieces],
    row_piece int64 [n_rows + 1])."""
    if chunk <= 0:
        raise ValueError("chunk must be positive")
    dev = rowptr.device
    counts = rowptr[1:] - rowptr[:-1]
    per_row = (counts + (chunk - 1)) // chunk
    row_piece = torch.zeros(rowptr.numel(), dtype=torch.int64, device=dev)
    row_piece[1:] = torch.cumsum(per_row, 0)
    n_pieces = int(row_piece[-1])
    piece_row = torch.repeat_interleave(torch.arange(counts.numel(), device=dev), per_row)
    k_in_row = torch.arange(n_pieces, device=dev) - row_piece[:-1][piece_row]
    start = rowptr[:-1][piece_row] + k_in_row * chunk
    piece_ptr = torch.empty(n_pieces + 1, dtype=torch.int64, device=dev)
    piece_ptr[:-1] = start
    piece_ptr[-1] = rowptr[-1]
    return piece_ptr, piece_row.to(torch.int32), row_piece


def transpose_permutation(rowptr, col, n_cols):
    """perm int64 [nnz]: entry i of the transposed operator (as built by transpose_csr) is entry
    perm[i] of the operator, so that valuesT = values[perm]."""
    n_rows = int(rowptr.numel()) - 1
    counts = rowptr[1:] - rowptr[:-1]
    rows = torch.repeat_interleave(torch.arange(n_rows, device=rowptr.device), counts)
    key = col.to(torch.int64) * n_rows + rows
    return torch.sort(key, stable=True).indices
