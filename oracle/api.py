"""numpy front end of the C oracle (oracle/sylvie_oracle.c).

Each wrapper only checks shapes/dtypes and forwards pointers; all arithmetic is
in the C file.  Arrays are C-contiguous numpy arrays; float data is float32.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sylvie_oracle.c")
_SO = os.path.join(_HERE, "libsylvie_oracle.so")
_lock = threading.Lock()
_lib = None

__all__ = [
    "build", "words_per_row", "uniform24", "quantize_1bit", "dequantize_1bit_fwd",
    "dequantize_1bit_bwd", "gcn_operator", "mean_weights", "aggregate_fwd", "aggregate_bwd",
    "aggregate_bwd_rows", "transform_fwd", "transform_bwd", "num_threads", "set_num_threads",
    "words_per_row_bits", "quantize_bbit", "dequantize_bbit_fwd", "dequantize_bbit_bwd",
    "words_per_row_fp16", "convert_fp16", "recover_fp16_fwd", "recover_fp16_bwd",
    "softmax_xent", "sum_gradients", "sgd_update",
    "row_dot", "edge_softmax_fwd", "sddmm", "edge_softmax_bwd", "segment_sum", "column_sum",
    "rank1_add",
    "halo_set", "relabel_columns", "rows_in_owner", "recv_sets", "send_set", "transpose_csr",
    "scatter_segments",
]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no contraction, OpenMP over rows)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _L():
    global _lib
    with _lock:
        if _lib is None:
            build()
            lib = C.CDLL(_SO)
            lib.orc_uniform24.restype = C.c_uint32
            lib.orc_uniform24.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32]
            lib.orc_words_per_row.restype = C.c_int64
            lib.orc_words_per_row.argtypes = [C.c_int32]
            lib.orc_words_per_row_bits.restype = C.c_int64
            lib.orc_words_per_row_bits.argtypes = [C.c_int32, C.c_int32]
            lib.orc_words_per_row_fp16.restype = C.c_int64
            lib.orc_words_per_row_fp16.argtypes = [C.c_int32]
            lib.orc_softmax_xent.restype = C.c_double
            lib.orc_aggregate_bwd.restype = C.c_int
            lib.orc_num_threads.restype = C.c_int
            lib.orc_halo_set.restype = C.c_int64
            lib.orc_send_set.restype = C.c_int64
            _lib = lib
    return _lib


def _p(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _f32(a, name):
    if a.dtype != np.float32 or not a.flags.c_contiguous:
        raise TypeError(f"{name}: need C-contiguous float32")
    return a


def _chk(a, dtype, name):
    if a.dtype != dtype or not a.flags.c_contiguous:
        raise TypeError(f"{name}: need C-contiguous {np.dtype(dtype).name}")
    return a


def num_threads() -> int:
    return int(_L().orc_num_threads())


def set_num_threads(n: int) -> None:
    """Threads for the row loops from now on (a timing knob; results do not depend on it)."""
    _L().orc_set_num_threads(C.c_int(int(n)))


def words_per_row(d: int) -> int:
    return int(_L().orc_words_per_row(int(d)))


def uniform24(seed: int, stream: int, row: int, col: int) -> int:
    return int(_L().orc_uniform24(C.c_uint64(seed), C.c_uint32(stream), C.c_uint32(row),
                                  C.c_uint32(col)))


def quantize_1bit(src, d, n_rows, seed, stream, idx=None, row_offset=0, wire_row0=0):
    """-> (packed uint64 [n_rows, W], scale f32 [n_rows], zero f32 [n_rows]).
    wire_row0: index of the first of these rows in the exchange they belong to."""
    _f32(src, "src")
    ld = src.shape[1]
    W = words_per_row(d)
    packed = np.empty((n_rows, W), np.uint64)
    scale = np.empty(n_rows, np.float32)
    zero = np.empty(n_rows, np.float32)
    if idx is not None:
        _chk(idx, np.int32, "idx")
    _L().orc_quantize_1bit(_p(src), C.c_int64(ld), C.c_int32(d), _p(idx), C.c_int64(row_offset),
                           C.c_int64(n_rows), C.c_uint64(seed), C.c_uint32(stream),
                           C.c_int64(wire_row0), _p(packed), _p(scale), _p(zero))
    return packed, scale, zero


def dequantize_1bit_fwd(packed, scale, zero, d, dst, row_offset):
    """dst[row_offset + i, :d] = dequantised wire row i (in place)."""
    _chk(packed, np.uint64, "packed"); _f32(scale, "scale"); _f32(zero, "zero"); _f32(dst, "dst")
    n = packed.shape[0]
    _L().orc_dequantize_1bit_fwd(_p(packed), _p(scale), _p(zero), C.c_int64(n), C.c_int32(d),
                                 _p(dst), C.c_int64(dst.shape[1]), C.c_int64(row_offset))


def dequantize_1bit_bwd(packed, scale, zero, d, J, dst_row):
    """J[dst_row[i], :d] += dequantised wire row i, ascending i (in place)."""
    _chk(packed, np.uint64, "packed"); _f32(scale, "scale"); _f32(zero, "zero"); _f32(J, "J")
    _chk(dst_row, np.int32, "dst_row")
    n = packed.shape[0]
    _L().orc_dequantize_1bit_bwd(_p(packed), _p(scale), _p(zero), C.c_int64(n), C.c_int32(d),
                                 _p(J), C.c_int64(J.shape[1]), _p(dst_row))


def words_per_row_bits(d: int, bits: int) -> int:
    return int(_L().orc_words_per_row_bits(int(d), int(bits)))


def _bits_ok(bits):
    if bits not in (1, 2, 4, 8):
        raise ValueError("bits must be 1, 2, 4 or 8")


def quantize_bbit(src, d, n_rows, bits, seed, stream, idx=None, row_offset=0, wire_row0=0):
    """b-bit codes -> (packed uint64 [n_rows, ceil(d*bits/64)], scale f32, zero f32)."""
    _bits_ok(bits)
    _f32(src, "src")
    W = words_per_row_bits(d, bits)
    packed = np.empty((n_rows, W), np.uint64)
    scale = np.empty(n_rows, np.float32)
    zero = np.empty(n_rows, np.float32)
    if idx is not None:
        _chk(idx, np.int32, "idx")
    _L().orc_quantize_bbit(_p(src), C.c_int64(src.shape[1]), C.c_int32(d), _p(idx),
                           C.c_int64(row_offset), C.c_int64(n_rows), C.c_int32(bits),
                           C.c_uint64(seed), C.c_uint32(stream), C.c_int64(wire_row0), _p(packed),
                           _p(scale), _p(zero))
    return packed, scale, zero


def dequantize_bbit_fwd(packed, scale, zero, d, bits, dst, row_offset):
    _bits_ok(bits)
    _chk(packed, np.uint64, "packed"); _f32(scale, "scale"); _f32(zero, "zero"); _f32(dst, "dst")
    _L().orc_dequantize_bbit_fwd(_p(packed), _p(scale), _p(zero), C.c_int64(packed.shape[0]),
                                 C.c_int32(d), C.c_int32(bits), _p(dst), C.c_int64(dst.shape[1]),
                                 C.c_int64(row_offset))


def dequantize_bbit_bwd(packed, scale, zero, d, bits, J, dst_row):
    _bits_ok(bits)
    _chk(packed, np.uint64, "packed"); _f32(scale, "scale"); _f32(zero, "zero"); _f32(J, "J")
    _chk(dst_row, np.int32, "dst_row")
    _L().orc_dequantize_bbit_bwd(_p(packed), _p(scale), _p(zero), C.c_int64(packed.shape[0]),
                                 C.c_int32(d), C.c_int32(bits), _p(J), C.c_int64(J.shape[1]),
                                 _p(dst_row))


def words_per_row_fp16(d: int) -> int:
    return int(_L().orc_words_per_row_fp16(int(d)))


def convert_fp16(src, d, n_rows, idx=None, row_offset=0):
    """-> wire uint16 [n_rows, 4*ceil(d/4)]: binary16 bit patterns, zero padded."""
    _f32(src, "src")
    if idx is not None:
        _chk(idx, np.int32, "idx")
    wire = np.empty((n_rows, 4 * words_per_row_fp16(d)), np.uint16)
    _L().orc_convert_fp16(_p(src), C.c_int64(src.shape[1]), C.c_int32(d), _p(idx),
                          C.c_int64(row_offset), C.c_int64(n_rows), _p(wire))
    return wire


def recover_fp16_fwd(wire, d, dst, row_offset):
    _chk(wire, np.uint16, "wire"); _f32(dst, "dst")
    _L().orc_recover_fp16_fwd(_p(wire), C.c_int64(wire.shape[0]), C.c_int32(d), _p(dst),
                              C.c_int64(dst.shape[1]), C.c_int64(row_offset))


def recover_fp16_bwd(wire, d, J, dst_row):
    _chk(wire, np.uint16, "wire"); _f32(J, "J"); _chk(dst_row, np.int32, "dst_row")
    _L().orc_recover_fp16_bwd(_p(wire), C.c_int64(wire.shape[0]), C.c_int32(d), _p(J),
                              C.c_int64(J.shape[1]), _p(dst_row))


def gcn_operator(rowptr, col, deg, n_in):
    """-> (rowptr', col', w) of D^-1/2 (A + I) D^-1/2 restricted to the inner rows."""
    _chk(rowptr, np.int64, "rowptr"); _chk(col, np.int32, "col"); _chk(deg, np.int32, "deg")
    nnz = int(rowptr[n_in])
    orp = np.empty(n_in + 1, np.int64)
    ocol = np.empty(nnz + n_in, np.int32)
    ow = np.empty(nnz + n_in, np.float32)
    _L().orc_gcn_operator(_p(rowptr), _p(col), _p(deg), C.c_int64(n_in), _p(orp), _p(ocol),
                          _p(ow))
    return orp, ocol, ow


def mean_weights(rowptr, n_in):
    _chk(rowptr, np.int64, "rowptr")
    w = np.empty(int(rowptr[n_in]), np.float32)
    _L().orc_mean_weights(_p(rowptr), C.c_int64(n_in), _p(w))
    return w


def aggregate_fwd(rowptr, col, w, X, d, want_S=False):
    """-> Z [n_rows, d] (and S, the sum of |terms|, if want_S)."""
    _chk(rowptr, np.int64, "rowptr"); _chk(col, np.int32, "col"); _f32(w, "w"); _f32(X, "X")
    n = rowptr.shape[0] - 1
    Z = np.empty((n, d), np.float32)
    S = np.empty((n, d), np.float32) if want_S else None
    _L().orc_aggregate_fwd(_p(rowptr), _p(col), _p(w), C.c_int64(n), _p(X),
                           C.c_int64(X.shape[1]), C.c_int32(d), _p(Z), C.c_int64(d), _p(S),
                           C.c_int64(d))
    return (Z, S) if want_S else Z


def aggregate_bwd(rowptr, col, w, n_cols, dZ, d, want_S=False):
    """-> dX [n_cols, d] = A^T dZ (and S if want_S)."""
    _chk(rowptr, np.int64, "rowptr"); _chk(col, np.int32, "col"); _f32(w, "w"); _f32(dZ, "dZ")
    n = rowptr.shape[0] - 1
    dX = np.empty((n_cols, d), np.float32)
    S = np.empty((n_cols, d), np.float32) if want_S else None
    rc = _L().orc_aggregate_bwd(_p(rowptr), _p(col), _p(w), C.c_int64(n), C.c_int64(n_cols),
                                _p(dZ), C.c_int64(dZ.shape[1]), C.c_int32(d), _p(dX),
                                C.c_int64(d), _p(S), C.c_int64(d))
    if rc != 0:
        raise MemoryError("oracle aggregate_bwd: out of memory")
    return (dX, S) if want_S else dX


def aggregate_bwd_rows(rowptr, col, w, dZ, d, sel):
    """Rows sel (ascending, distinct) of A^T dZ -> (out [n_sel, d], S [n_sel, d])."""
    _chk(rowptr, np.int64, "rowptr"); _chk(col, np.int32, "col"); _f32(w, "w"); _f32(dZ, "dZ")
    _chk(sel, np.int32, "sel")
    n = rowptr.shape[0] - 1
    out = np.empty((sel.shape[0], d), np.float32)
    S = np.empty((sel.shape[0], d), np.float32)
    _L().orc_aggregate_bwd_rows(_p(rowptr), _p(col), _p(w), C.c_int64(n), _p(dZ),
                                C.c_int64(dZ.shape[1]), C.c_int32(d), _p(sel),
                                C.c_int64(sel.shape[0]), _p(out), _p(S))
    return out, S


def transform_fwd(A1, Wm, relu, A2=None, want_S=False):
    """H = relu?(max([A1|A2] W, 0)) -> H [n, h] (and S if want_S)."""
    _f32(A1, "A1"); _f32(Wm, "W")
    n, k1 = A1.shape
    k2 = 0 if A2 is None else _f32(A2, "A2").shape[1]
    h = Wm.shape[1]
    assert Wm.shape[0] == k1 + k2
    H = np.empty((n, h), np.float32)
    S = np.empty((n, h), np.float32) if want_S else None
    _L().orc_transform_fwd(_p(A1), C.c_int64(k1), C.c_int32(k1), _p(A2), C.c_int64(k2),
                           C.c_int32(k2), _p(Wm), C.c_int32(h), C.c_int64(n), C.c_int(int(relu)),
                           _p(H), C.c_int64(h), None, _p(S))
    return (H, S) if want_S else H


def transform_bwd(A1, Wm, relu, H, J, A2=None, want_G=True, want_dA=True, want_S=False):
    """-> dict with G [(k1+k2), h], dA1 [n, k1], dA2 [n, k2] (and SG, SdA1, SdA2)."""
    _f32(A1, "A1"); _f32(Wm, "W"); _f32(H, "H"); _f32(J, "J")
    n, k1 = A1.shape
    k2 = 0 if A2 is None else _f32(A2, "A2").shape[1]
    h = Wm.shape[1]
    out = {}
    G = np.empty((k1 + k2, h), np.float32) if want_G else None
    dA1 = np.empty((n, k1), np.float32) if want_dA else None
    dA2 = np.empty((n, k2), np.float32) if (want_dA and k2) else None
    SG = np.empty((k1 + k2, h), np.float32) if (want_S and want_G) else None
    S1 = np.empty((n, k1), np.float32) if (want_S and want_dA) else None
    S2 = np.empty((n, k2), np.float32) if (want_S and want_dA and k2) else None
    _L().orc_transform_bwd(_p(A1), C.c_int64(k1), C.c_int32(k1), _p(A2), C.c_int64(k2),
                           C.c_int32(k2), _p(Wm), C.c_int32(h), C.c_int64(n), C.c_int(int(relu)),
                           _p(H), C.c_int64(h), _p(J), C.c_int64(J.shape[1]), _p(G), _p(SG),
                           _p(dA1), C.c_int64(k1), _p(dA2), C.c_int64(k2), _p(S1), _p(S2))
    out.update(G=G, dA1=dA1, dA2=dA2, SG=SG, SdA1=S1, SdA2=S2)
    return out


def softmax_xent(H, label, count, want_S=False):
    """-> (loss contribution of these rows, J f32 [n, C][, SJ])."""
    _f32(H, "H"); _chk(label, np.int32, "label")
    n, Cc = H.shape
    J = np.empty((n, Cc), np.float32)
    SJ = np.empty((n, Cc), np.float32) if want_S else None
    loss = _L().orc_softmax_xent(_p(H), C.c_int64(Cc), C.c_int64(n), C.c_int32(Cc), _p(label),
                                 C.c_double(float(count)), _p(J), C.c_int64(Cc), _p(SJ))
    return (float(loss), J, SJ) if want_S else (float(loss), J)


def sum_gradients(srcs):
    """Sum of equally shaped float32 arrays in list order, single precision."""
    for a in srcs:
        _f32(a, "src")
    dst = np.empty_like(srcs[0])
    ptrs = (C.c_void_p * len(srcs))(*[a.ctypes.data for a in srcs])
    _L().orc_sum_gradients(_p(dst), ptrs, C.c_int32(len(srcs)), C.c_int64(dst.size))
    return dst


def sgd_update(W, G, eta):
    """In place: W = W - eta * G (single precision)."""
    _f32(W, "W"); _f32(G, "G")
    _L().orc_sgd_update(_p(W), _p(G), C.c_int64(W.size), C.c_float(eta))


def row_dot(P, a, n=None):
    _f32(P, "P"); _f32(a, "a")
    n = P.shape[0] if n is None else n
    out = np.empty(n, np.float32)
    _L().orc_row_dot(_p(P), C.c_int64(P.shape[1]), C.c_int64(n), C.c_int32(a.shape[0]), _p(a), _p(out))
    return out


def edge_softmax_fwd(rowptr, col, s_dst, s_src, slope):
    _chk(rowptr, np.int64, "rowptr"); _chk(col, np.int32, "col"); _f32(s_dst, "s_dst"); _f32(s_src, "s_src")
    n = rowptr.shape[0] - 1
    alpha = np.zeros(int(rowptr[-1]), np.float32)
    _L().orc_edge_softmax_fwd(_p(rowptr), _p(col), C.c_int64(n), _p(s_dst), _p(s_src), C.c_float(slope),
                              _p(alpha))
    return alpha


def sddmm(rowptr, col, A, Bm, F, want_S=False):
    _chk(rowptr, np.int64, "rowptr"); _chk(col, np.int32, "col"); _f32(A, "A"); _f32(Bm, "B")
    n = rowptr.shape[0] - 1
    out = np.zeros(int(rowptr[-1]), np.float32)
    S = np.zeros_like(out) if want_S else None
    _L().orc_sddmm(_p(rowptr), _p(col), C.c_int64(n), _p(A), C.c_int64(A.shape[1]), _p(Bm),
                   C.c_int64(Bm.shape[1]), C.c_int32(F), _p(out), _p(S))
    return (out, S) if want_S else out


def edge_softmax_bwd(rowptr, col, alpha, dalpha, s_dst, s_src, slope, want_S=False):
    _chk(rowptr, np.int64, "rowptr"); _chk(col, np.int32, "col")
    for a_, nm in ((alpha, "alpha"), (dalpha, "dalpha"), (s_dst, "s_dst"), (s_src, "s_src")):
        _f32(a_, nm)
    n = rowptr.shape[0] - 1
    de = np.zeros(int(rowptr[-1]), np.float32)
    S = np.zeros_like(de) if want_S else None
    _L().orc_edge_softmax_bwd(_p(rowptr), _p(col), C.c_int64(n), _p(alpha), _p(dalpha), _p(s_dst),
                              _p(s_src), C.c_float(slope), _p(de), _p(S))
    return (de, S) if want_S else de


def segment_sum(rowptr, vals, want_S=False):
    _chk(rowptr, np.int64, "rowptr"); _f32(vals, "vals")
    n = rowptr.shape[0] - 1
    out = np.empty(n, np.float32)
    S = np.empty(n, np.float32) if want_S else None
    _L().orc_segment_sum(_p(rowptr), C.c_int64(n), _p(vals), _p(out), _p(S))
    return (out, S) if want_S else out


def column_sum(rowptr, col, n_cols, vals, want_S=False):
    _chk(rowptr, np.int64, "rowptr"); _chk(col, np.int32, "col"); _f32(vals, "vals")
    n = rowptr.shape[0] - 1
    out = np.empty(n_cols, np.float32)
    S = np.empty(n_cols, np.float32) if want_S else None
    _L().orc_column_sum(_p(rowptr), _p(col), C.c_int64(n), C.c_int64(n_cols), _p(vals), _p(out), _p(S))
    return (out, S) if want_S else out


def rank1_add(X, n, s, a):
    """In place: X[i, :F] += s[i] * a for i < n (single precision)."""
    _f32(X, "X"); _f32(s, "s"); _f32(a, "a")
    _L().orc_rank1_add(_p(X), C.c_int64(X.shape[1]), C.c_int64(n), C.c_int32(a.shape[0]), _p(s), _p(a))


# ---- Graph Engine set-up (Alg. 1, the lines before the epoch loop) -------------------

def halo_set(rowptr, gcol, n_in, owner, part):
    """-> (halo_gid int32 ascending, pos int32 [n_nodes], n_inner): V_HALO,n and the local numbering."""
    _chk(rowptr, np.int64, "rowptr"); _chk(gcol, np.int32, "gcol"); _chk(owner, np.int32, "owner")
    n_nodes = owner.shape[0]
    pos = np.empty(n_nodes, np.int32)
    halo = np.empty(n_nodes, np.int32)
    n_inner = C.c_int64(0)
    n_halo = _L().orc_halo_set(_p(rowptr), _p(gcol), C.c_int64(n_in), _p(owner), C.c_int64(n_nodes),
                               C.c_int32(part), _p(pos), _p(halo), C.byref(n_inner))
    return halo[:n_halo].copy(), pos, int(n_inner.value)


def relabel_columns(gcol, pos):
    _chk(gcol, np.int32, "gcol"); _chk(pos, np.int32, "pos")
    col = np.empty(gcol.shape[0], np.int32)
    _L().orc_relabel_columns(_p(gcol), C.c_int64(gcol.shape[0]), _p(pos), _p(col))
    return col


def rows_in_owner(owner, n_parts):
    """-> (row_of int32 [n_nodes], part_ptr int64 [n_parts + 1])."""
    _chk(owner, np.int32, "owner")
    row_of = np.empty(owner.shape[0], np.int32)
    part_ptr = np.empty(n_parts + 1, np.int64)
    _L().orc_rows_in_owner(_p(owner), C.c_int64(owner.shape[0]), C.c_int32(n_parts), _p(row_of), _p(part_ptr))
    return row_of, part_ptr


def recv_sets(halo_gid, owner, row_of, n_parts):
    """-> (R_ptr int64 [n_parts + 1], R_halo int32, R_row int32): R_k = V_HALO,n & V_k."""
    _chk(halo_gid, np.int32, "halo_gid"); _chk(owner, np.int32, "owner"); _chk(row_of, np.int32, "row_of")
    n = halo_gid.shape[0]
    R_ptr = np.empty(n_parts + 1, np.int64)
    R_halo = np.empty(n, np.int32); R_row = np.empty(n, np.int32)
    _L().orc_recv_sets(_p(halo_gid), C.c_int64(n), _p(owner), _p(row_of), C.c_int32(n_parts),
                       _p(R_ptr), _p(R_halo), _p(R_row))
    return R_ptr, R_halo, R_row


def send_set(peer_halo, owner, row_of, part):
    """-> S_row int32: S_k = V_n & V_HALO,k as rows of partition `part`'s inner block."""
    _chk(peer_halo, np.int32, "peer_halo"); _chk(owner, np.int32, "owner"); _chk(row_of, np.int32, "row_of")
    S = np.empty(peer_halo.shape[0], np.int32)
    n = _L().orc_send_set(_p(peer_halo), C.c_int64(peer_halo.shape[0]), _p(owner), _p(row_of),
                          C.c_int32(part), _p(S))
    return S[:n].copy()


def transpose_csr(rowptr, col, w, n_cols):
    """-> (rowptrT int64, colT int32, wT float32 | None, perm int64)."""
    _chk(rowptr, np.int64, "rowptr"); _chk(col, np.int32, "col")
    if w is not None:
        _f32(w, "w")
    n_rows, nnz = rowptr.shape[0] - 1, col.shape[0]
    rowptrT = np.empty(n_cols + 1, np.int64)
    colT = np.empty(nnz, np.int32); perm = np.empty(nnz, np.int64)
    wT = np.empty(nnz, np.float32) if w is not None else None
    _L().orc_transpose_csr(_p(rowptr), _p(col), _p(w), C.c_int64(n_rows), C.c_int64(n_cols),
                           _p(rowptrT), _p(colT), _p(wT), _p(perm))
    return rowptrT, colT, wT, perm


def scatter_segments(dst_row, n_dst):
    """-> (seg_ptr int64 [n_dst + 1], seg_rows int32 [n])."""
    _chk(dst_row, np.int32, "dst_row")
    seg_ptr = np.empty(n_dst + 1, np.int64)
    seg_rows = np.empty(dst_row.shape[0], np.int32)
    _L().orc_scatter_segments(_p(dst_row), C.c_int64(dst_row.shape[0]), C.c_int64(n_dst), _p(seg_ptr), _p(seg_rows))
    return seg_ptr, seg_rows
