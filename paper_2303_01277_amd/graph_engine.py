"""One-off set-up of a partition (the "Graph Engine" step, Sec. 3.2; Alg. 1 lines 3-7).

Builds, once per graph, the index structures the kernels consume: the HALO set and the
local numbering of a partition, its receive / send sets, the normalised operator
(Sec. 3.4), its transpose as a CSR of its own, the plan that cuts long rows into tasks,
and the scatter segments of the backward dequantizer.  Everything runs in the library's own
kernels (GPU tensors only); this module allocates the outputs and the workspaces and slices
them to the counts the library reports.  None of this is on the per-layer hot path.
"""
from __future__ import annotations

import torch

from . import binding as B


def _workspace(n, dev):
    return torch.empty(B.sylvie_graph_workspace_bytes(n) // 8 + 1, dtype=torch.int64, device=dev)


def local_index(gcol, n_in, owner, part):
    """V_HALO,n and the local numbering of partition `part` (Alg. 1, the HALO node set).

    gcol int32 [nnz]: global neighbour ids of the partition's inner rows; owner int32
    [n_nodes].  Returns (pos int32 [n_nodes], halo_gid int32 [n_halo] ascending, col int32
    [nnz]): pos[g] = local row of node g or -1, col = the adjacency in local rows.
    """
    dev = owner.device
    n_nodes, nnz = int(owner.numel()), int(gcol.numel())
    ws = _workspace(n_nodes, dev)
    pos = torch.empty(n_nodes, dtype=torch.int32, device=dev)
    # every named node is a distinct node that the partition does not own
    cap = max(0, min(nnz, n_nodes - n_in))
    halo_gid = torch.empty(max(cap, 1), dtype=torch.int32, device=dev)
    _, n_halo = B.sylvie_graph_local_index(gcol, nnz, n_in, owner, n_nodes, part, pos, halo_gid, cap, ws)
    col = torch.empty(nnz, dtype=torch.int32, device=dev)
    B.sylvie_graph_relabel_columns(gcol, nnz, pos, n_nodes, col, ws)
    return pos, halo_gid[:n_halo].clone(), col


def rows_in_owner(owner, n_parts):
    """(row_of int32 [n_nodes], part_ptr int64 [n_parts + 1]): every node's row in its owner's
    inner block (its rank among the owner's nodes, ascending id) and the partitions' sizes."""
    dev = owner.device
    n_nodes = int(owner.numel())
    row_of = torch.empty(n_nodes, dtype=torch.int32, device=dev)
    part_ptr = torch.empty(n_parts + 1, dtype=torch.int64, device=dev)
    B.sylvie_graph_rows_in_owner(owner, n_nodes, n_parts, row_of, part_ptr, _workspace(n_nodes, dev))
    return row_of, part_ptr


def recv_sets(halo_gid, owner, row_of, n_parts):
    """R_k = V_HALO,n & V_k for every k (Alg. 1, the receive sets): (R_ptr int64 [n_parts + 1],
    R_halo int32 [n_halo], R_row int32 [n_halo]); see sylvie_graph_recv_sets.  The rows partition
    n sends to k are R_row[R_ptr[n] : R_ptr[n+1]] of partition k's result."""
    dev = owner.device
    n_halo = int(halo_gid.numel())
    R_ptr = torch.empty(n_parts + 1, dtype=torch.int64, device=dev)
    R_halo = torch.empty(n_halo, dtype=torch.int32, device=dev)
    R_row = torch.empty(n_halo, dtype=torch.int32, device=dev)
    B.sylvie_graph_recv_sets(halo_gid if n_halo else None, n_halo, owner, row_of, int(owner.numel()), n_parts,
                             R_ptr, R_halo if n_halo else None, R_row if n_halo else None, _workspace(n_halo, dev))
    return R_ptr, R_halo, R_row


def gcn_operator(rowptr, col, deg, n_in):
    """Rows of D^-1/2 (A + I) D^-1/2 for the inner nodes of a partition (Sec. 3.4).

    rowptr/col: adjacency of the inner rows over all local rows (inner + halo), no
    self loops, columns ascending.  deg[r]: degree of local row r in the whole
    graph, self loop not counted.  Returns (rowptr', col', w) with the self loop
    (r, r) merged in column order and w = 1/sqrt((deg_r + 1)(deg_c + 1)) evaluated
    in float64, rounded once to float32 (sylvie_graph_gcn_operator).
    """
    dev = rowptr.device
    nnz, n_cols = int(col.numel()), int(deg.numel())
    rowptr_out = torch.empty(n_in + 1, dtype=torch.int64, device=dev)
    col_out = torch.empty(max(1, nnz + n_in), dtype=torch.int32, device=dev)
    w_out = torch.empty(max(1, nnz + n_in), dtype=torch.float32, device=dev)
    B.sylvie_graph_gcn_operator(rowptr, col if nnz else None, deg, n_in, n_cols, nnz, rowptr_out, col_out, w_out,
                                _workspace(1, dev))
    return rowptr_out, col_out[: nnz + n_in], w_out[: nnz + n_in]


def mean_operator(rowptr, col, n_in):
    """GraphSAGE mean aggregator: every entry of row r weighs 1/len(r) (sylvie_graph_mean_weights)."""
    nnz = int(col.numel())
    w = torch.empty(max(1, nnz), dtype=torch.float32, device=rowptr.device)
    B.sylvie_graph_mean_weights(rowptr, n_in, nnz, w, _workspace(1, rowptr.device))
    return rowptr, col, w[:nnz]


def transpose_csr(rowptr, col, w, n_cols, want_perm=False):
    """CSR of the transposed operator: n_cols rows; entries of a row in ascending
    original-row order.  Returns (rowptrT int64, colT int32, wT float32) and, with
    want_perm, perm int64 [nnz]: entry i of the transpose is entry perm[i] of the
    operator (valuesT = values[perm])."""
    dev = rowptr.device
    n_rows, nnz = int(rowptr.numel()) - 1, int(col.numel())
    rowptrT = torch.empty(n_cols + 1, dtype=torch.int64, device=dev)
    colT = torch.empty(nnz, dtype=torch.int32, device=dev)
    wT = None if w is None else torch.empty(nnz, dtype=torch.float32, device=dev)
    perm = torch.empty(nnz, dtype=torch.int64, device=dev) if want_perm else None
    B.sylvie_graph_transpose_csr(rowptr, col if nnz else None, w if nnz else None, n_rows, n_cols, nnz, rowptrT,
                                 colT if nnz else None, wT if nnz else None, perm if nnz else None,
                                 _workspace(nnz, dev))
    return (rowptrT, colT, wT, perm) if want_perm else (rowptrT, colT, wT)


def long_row_plan(rowptr, chunk, row_begin=0, row_end=None, nnz=None):
    """Rows longer than `chunk` entries (absolute indices, optionally only those in
    [row_begin, row_end)) and the prefix sum of their task counts (sylvie_graph_long_row_plan).
    Returns (long_rows int32 [n_long], long_ptr int64 [n_long + 1], n_tasks).  nnz: entries of
    the row range if the caller knows them (bounds the number of long rows without a read-back)."""
    if chunk <= 0 or chunk % 64:
        raise ValueError("chunk must be a positive multiple of 64")
    dev = rowptr.device
    n = int(rowptr.numel()) - 1
    hi = n if row_end is None else row_end
    n_rows = hi - row_begin
    cap = n_rows if nnz is None else min(n_rows, nnz // chunk + 1)
    long_rows = torch.empty(max(1, cap), dtype=torch.int32, device=dev)
    long_ptr = torch.empty(cap + 1, dtype=torch.int64, device=dev)
    n_long, n_tasks = B.sylvie_graph_long_row_plan(rowptr, row_begin, n_rows, chunk, long_rows, long_ptr, cap,
                                                   _workspace(n_rows, dev))
    return long_rows[:n_long], long_ptr[: n_long + 1], n_tasks


def rows_by_length(rowptr, row_begin=0, row_end=None):
    """Processing order of the rows [row_begin, row_end) of a CSR for the aggregation kernels:
    longest row first, ties in index order (sylvie_graph_rows_by_length).  Returns int32
    [row_end - row_begin], a permutation of [0, row_end - row_begin) (indices relative to row_begin)."""
    dev = rowptr.device
    n = int(rowptr.numel()) - 1
    hi = n if row_end is None else row_end
    n_rows = hi - row_begin
    order = torch.empty(max(1, n_rows), dtype=torch.int32, device=dev)
    B.sylvie_graph_rows_by_length(rowptr, row_begin, n_rows, order, _workspace(n_rows, dev))
    return order[:n_rows]


def scatter_segments_dense(dst_row, n_dst):
    """Wire rows grouped by destination row, one (possibly empty) segment for every
    destination row 0 .. n_dst - 1: returns (seg_ptr int64 [n_dst + 1], seg_rows int32 [n]);
    destination r receives wire rows seg_rows[seg_ptr[r] : seg_ptr[r+1]], ascending."""
    dev = dst_row.device
    n = int(dst_row.numel())
    seg_ptr = torch.empty(n_dst + 1, dtype=torch.int64, device=dev)
    seg_rows = torch.empty(n, dtype=torch.int32, device=dev)
    B.sylvie_graph_scatter_segments(dst_row if n else None, n, n_dst, seg_ptr, seg_rows if n else None,
                                    _workspace(n, dev))
    return seg_ptr, seg_rows


def scatter_segments(dst_row, n_dst=None):
    """Group wire rows by destination row for the backward dequantizer, destinations
    without wire rows left out.

    dst_row int32 [n]: destination of wire row i.  Returns (seg_ptr int64 [m + 1],
    seg_rows int32 [n], dst_ids int32 [m]): destination dst_ids[k] receives wire
    rows seg_rows[seg_ptr[k] : seg_ptr[k+1]], ascending.
    """
    if n_dst is None:
        n_dst = int(dst_row.max()) + 1 if dst_row.numel() else 1
    dense_ptr, seg_rows = scatter_segments_dense(dst_row, n_dst)
    dst_ids = torch.nonzero(dense_ptr[1:] > dense_ptr[:-1]).flatten()
    seg_ptr = torch.cat([dense_ptr[dst_ids], dense_ptr[-1:]])
    return seg_ptr, seg_rows, dst_ids.to(torch.int32)


def piece_table(rowptr, chunk, nnz=None):
    """Cuts every row's entries into pieces of at most `chunk` consecutive entries (rows without
    entries get none; sylvie_graph_piece_table).  Returns (piece_ptr int64 [n_pieces + 1], piece_row
    int32 [n_pieces], row_piece int64 [n_rows + 1]).  nnz: the number of entries, if the caller
    knows it (otherwise it is read back from the row pointer)."""
    if chunk <= 0:
        raise ValueError("chunk must be positive")
    dev = rowptr.device
    n_rows = int(rowptr.numel()) - 1
    if nnz is None:
        nnz = int(rowptr[-1])
    cap = n_rows + nnz // chunk
    row_piece = torch.empty(n_rows + 1, dtype=torch.int64, device=dev)
    piece_ptr = torch.empty(cap + 1, dtype=torch.int64, device=dev)
    piece_row = torch.empty(max(1, cap), dtype=torch.int32, device=dev)
    n_pieces = B.sylvie_graph_piece_table(rowptr, n_rows, chunk, row_piece, piece_ptr, piece_row, cap,
                                          _workspace(n_rows, dev))
    return piece_ptr[: n_pieces + 1], piece_row[:n_pieces], row_piece
