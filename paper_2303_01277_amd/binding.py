"""ctypes binding of libsylvie.so: one wrapper per entry point of include/sylvie.h.

The wrappers take torch tensors that already live on the GPU, check nothing but
device and dtype, and pass raw pointers, sizes and the current HIP stream.  There
is no CPU path: if the library is not built, or a tensor is not on the GPU, the
call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

from .build import library_path

_lib = None


class SylvieError(RuntimeError):
    pass


def lib():
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise SylvieError(
                f"{path} is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "(there is no CPU fallback)")
        L = C.CDLL(path)
        L.sylvie_version.restype = C.c_int32
        L.sylvie_status_string.restype = C.c_char_p
        L.sylvie_status_string.argtypes = [C.c_int32]
        L.sylvie_last_error.restype = C.c_char_p
        L.sylvie_wire_row_words.restype = C.c_int64
        L.sylvie_wire_row_words.argtypes = [C.c_int32]
        L.sylvie_wire_row_words_bits.restype = C.c_size_t
        L.sylvie_wire_row_words_bits.argtypes = [C.c_int32, C.c_int32]
        L.sylvie_scaled_column_sum_workspace_bytes.restype = C.c_size_t
        L.sylvie_scaled_column_sum_workspace_bytes.argtypes = [C.c_int64, C.c_int32]
        L.sylvie_edge_softmax_workspace_bytes.restype = C.c_size_t
        L.sylvie_edge_softmax_workspace_bytes.argtypes = [C.c_int64, C.c_int64]
        L.sylvie_edge_softmax_heads_workspace_bytes.restype = C.c_size_t
        L.sylvie_edge_softmax_heads_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32]
        L.sylvie_graph_workspace_bytes.restype = C.c_size_t
        L.sylvie_graph_workspace_bytes.argtypes = [C.c_int64]
        L.sylvie_transform_bwd_workspace_bytes.restype = C.c_size_t
        L.sylvie_transform_bwd_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32,
                                                           C.c_int64]
        for name in ("sylvie_quantize_1bit_fwd", "sylvie_quantize_1bit_bwd",
                     "sylvie_dequantize_1bit_fwd", "sylvie_dequantize_1bit_bwd",
                     "sylvie_quantize_bbit_fwd", "sylvie_quantize_bbit_bwd",
                     "sylvie_dequantize_bbit_fwd", "sylvie_dequantize_bbit_bwd",
                     "sylvie_aggregate_csr_fwd", "sylvie_aggregate_csr_bwd",
                     "sylvie_aggregate_csr_fwd_noalloc",
                     "sylvie_aggregate_csr_fwd_wire", "sylvie_aggregate_csr_bwd_quantize",
                     "sylvie_aggregate_csr_bwd_integrate",
                     "sylvie_aggregate_csr_fwd_wire_bbit", "sylvie_aggregate_csr_bwd_quantize_bbit",
                     "sylvie_aggregate_csr_bwd_integrate_bbit",
                     "sylvie_transform_fwd", "sylvie_transform_bwd", "sylvie_softmax_xent",
                     "sylvie_sum_gradients", "sylvie_sgd_update", "sylvie_row_dot",
                     "sylvie_edge_softmax_fwd", "sylvie_sddmm", "sylvie_edge_softmax_bwd",
                     "sylvie_segment_sum", "sylvie_permute_f32", "sylvie_rank1_add",
                     "sylvie_scaled_column_sum",
                     "sylvie_relu_fwd", "sylvie_relu_bwd",
                     "sylvie_row_dot_heads", "sylvie_edge_softmax_fwd_heads", "sylvie_sddmm_heads",
                     "sylvie_edge_softmax_bwd_heads", "sylvie_segment_sum_heads",
                     "sylvie_scaled_column_sum_heads", "sylvie_aggregate_csr_attention",
                     "sylvie_rank1_add_heads", "sylvie_aggregate_csr_attention_sddmm",
                     "sylvie_seed_offset_source",
                     "sylvie_aggregate_csr_attention_sddmm_supported",
                     "sylvie_graph_local_index", "sylvie_graph_relabel_columns",
                     "sylvie_graph_rows_in_owner", "sylvie_graph_recv_sets",
                     "sylvie_graph_transpose_csr", "sylvie_graph_scatter_segments",
                     "sylvie_graph_gcn_operator", "sylvie_graph_mean_weights",
                     "sylvie_graph_long_row_plan", "sylvie_graph_piece_table",
                     "sylvie_graph_rows_by_length"):
            getattr(L, name).restype = C.c_int32
        _lib = L
    return _lib


def _ptr(t, dtype=None, name="tensor"):
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda:
        raise SylvieError(f"{name}: expected a GPU tensor (there is no CPU path)")
    if dtype is not None and t.dtype != dtype:
        raise SylvieError(f"{name}: expected {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc):
    if rc != 0:
        L = lib()
        raise SylvieError(f"{L.sylvie_status_string(rc).decode()} ({rc}): "
                          f"{L.sylvie_last_error().decode()}")


def sylvie_version() -> int:
    return int(lib().sylvie_version())


def sylvie_wire_row_words(d: int) -> int:
    return int(lib().sylvie_wire_row_words(int(d)))


def _quantize(fn, src, ld_src, d, idx, row_offset, n_rows, seed, stream_id, wire_out, ld_wire):
    _check(fn(_ptr(src, torch.float32, "src"), C.c_int64(ld_src), C.c_int32(d),
              _ptr(idx, torch.int32, "idx"), C.c_int64(row_offset), C.c_int64(n_rows),
              C.c_uint64(seed & (2**64 - 1)), C.c_uint32(stream_id & 0xFFFFFFFF),
              _ptr(wire_out, torch.int64, "wire_out"), C.c_int64(ld_wire), _stream()))


def sylvie_quantize_1bit_fwd(src, ld_src, d, idx, row_offset, n_rows, seed, stream_id, wire_out,
                             ld_wire=0):
    """wire_out is an int64 tensor holding the uint64 wire words (torch has no uint64 kernels);
    ld_wire = words from one wire row to the next, 0 = packed."""
    _quantize(lib().sylvie_quantize_1bit_fwd, src, ld_src, d, idx, row_offset, n_rows, seed,
              stream_id, wire_out, ld_wire)


def sylvie_quantize_1bit_bwd(src, ld_src, d, idx, row_offset, n_rows, seed, stream_id, wire_out,
                             ld_wire=0):
    _quantize(lib().sylvie_quantize_1bit_bwd, src, ld_src, d, idx, row_offset, n_rows, seed,
              stream_id, wire_out, ld_wire)


def sylvie_wire_row_words_bits(d: int, bits: int) -> int:
    return int(lib().sylvie_wire_row_words_bits(int(d), int(bits)))


def _quantize_bbit(fn, src, ld_src, d, idx, row_offset, n_rows, bits, seed, stream_id, wire_out):
    _check(fn(_ptr(src, torch.float32, "src"), C.c_int64(ld_src), C.c_int32(d),
              _ptr(idx, torch.int32, "idx"), C.c_int64(row_offset), C.c_int64(n_rows),
              C.c_int32(bits), C.c_uint64(seed & (2**64 - 1)), C.c_uint32(stream_id & 0xFFFFFFFF),
              _ptr(wire_out, torch.int64, "wire_out"), _stream()))


def sylvie_quantize_bbit_fwd(src, ld_src, d, idx, row_offset, n_rows, bits, seed, stream_id,
                             wire_out):
    _quantize_bbit(lib().sylvie_quantize_bbit_fwd, src, ld_src, d, idx, row_offset, n_rows, bits,
                   seed, stream_id, wire_out)


def sylvie_quantize_bbit_bwd(src, ld_src, d, idx, row_offset, n_rows, bits, seed, stream_id,
                             wire_out):
    _quantize_bbit(lib().sylvie_quantize_bbit_bwd, src, ld_src, d, idx, row_offset, n_rows, bits,
                   seed, stream_id, wire_out)


def sylvie_dequantize_bbit_fwd(wire, n_rows, d, bits, dst, ld_dst, row_offset):
    _check(lib().sylvie_dequantize_bbit_fwd(
        _ptr(wire, torch.int64, "wire"), C.c_int64(n_rows), C.c_int32(d), C.c_int32(bits),
        _ptr(dst, torch.float32, "dst"), C.c_int64(ld_dst), C.c_int64(row_offset), _stream()))


def sylvie_dequantize_bbit_bwd(wire, n_rows, d, bits, dst, ld_dst, seg_ptr, seg_rows, n_dst_rows,
                               dst_ids):
    _check(lib().sylvie_dequantize_bbit_bwd(
        _ptr(wire, torch.int64, "wire"), C.c_int64(n_rows), C.c_int32(d), C.c_int32(bits),
        _ptr(dst, torch.float32, "dst"), C.c_int64(ld_dst), _ptr(seg_ptr, torch.int64, "seg_ptr"),
        _ptr(seg_rows, torch.int32, "seg_rows"), C.c_int64(n_dst_rows),
        _ptr(dst_ids, torch.int32, "dst_ids"), _stream()))


def sylvie_dequantize_1bit_fwd(wire, n_rows, d, dst, ld_dst, row_offset, ld_wire=0):
    _check(lib().sylvie_dequantize_1bit_fwd(
        _ptr(wire, torch.int64, "wire"), C.c_int64(ld_wire), C.c_int64(n_rows), C.c_int32(d),
        _ptr(dst, torch.float32, "dst"), C.c_int64(ld_dst), C.c_int64(row_offset), _stream()))


def sylvie_dequantize_1bit_bwd(wire, n_rows, d, dst, ld_dst, seg_ptr, seg_rows, n_dst_rows,
                               dst_ids, ld_wire=0):
    _check(lib().sylvie_dequantize_1bit_bwd(
        _ptr(wire, torch.int64, "wire"), C.c_int64(ld_wire), C.c_int64(n_rows), C.c_int32(d),
        _ptr(dst, torch.float32, "dst"), C.c_int64(ld_dst), _ptr(seg_ptr, torch.int64, "seg_ptr"),
        _ptr(seg_rows, torch.int32, "seg_rows"), C.c_int64(n_dst_rows),
        _ptr(dst_ids, torch.int32, "dst_ids"), _stream()))


def _aggregate(fn, rowptr, col, w, row_scale, col_scale, n_rows, X, ld_x, d, Y, ld_y, addend,
               ld_addend, addend_rows, chunk, long_rows, long_ptr, n_long, n_tasks, workspace,
               row_order=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(fn(_ptr(rowptr, torch.int64, "rowptr"), _ptr(col, torch.int32, "col"),
              _ptr(w, torch.float32, "w"), _ptr(row_scale, torch.float32, "row_scale"),
              _ptr(col_scale, torch.float32, "col_scale"), C.c_int64(n_rows),
              _ptr(X, torch.float32, "X"), C.c_int64(ld_x), C.c_int32(d),
              _ptr(Y, torch.float32, "Y"), C.c_int64(ld_y), _ptr(addend, torch.float32, "addend"),
              C.c_int64(ld_addend), C.c_int64(addend_rows), _ptr(row_order, torch.int32, "row_order"),
              C.c_int32(chunk),
              _ptr(long_rows, torch.int32, "long_rows"), _ptr(long_ptr, torch.int64, "long_ptr"),
              C.c_int64(n_long), C.c_int64(n_tasks), _ptr(workspace, torch.float32, "workspace"),
              C.c_size_t(ws_bytes), _stream()))


def sylvie_aggregate_csr_fwd(rowptr, col, w, row_scale, col_scale, n_rows, X, ld_x, d, Y, ld_y,
                             addend=None, ld_addend=0, addend_rows=0, chunk=0, long_rows=None,
                             long_ptr=None, n_long=0, n_tasks=0, workspace=None, row_order=None):
    _aggregate(lib().sylvie_aggregate_csr_fwd, rowptr, col, w, row_scale, col_scale, n_rows, X,
               ld_x, d, Y, ld_y, addend, ld_addend, addend_rows, chunk, long_rows, long_ptr,
               n_long, n_tasks, workspace, row_order)


STATIC_SCRATCH_BYTES = 16 << 20


def sylvie_aggregate_csr_fwd_noalloc(rowptr, col, w, row_scale, col_scale, n_rows, X, ld_x, d, Y, ld_y,
                                     addend=None, ld_addend=0, addend_rows=0, chunk=0,
                                     long_rows=None, long_ptr=None, n_long=0, n_tasks=0, row_order=None):
    """sylvie_aggregate_csr_fwd with the long-row partial sums in the library's built-in scratch
    (n_tasks * d * 4 <= STATIC_SCRATCH_BYTES); allocates nothing."""
    _check(lib().sylvie_aggregate_csr_fwd_noalloc(
        _ptr(rowptr, torch.int64, "rowptr"), _ptr(col, torch.int32, "col"),
        _ptr(w, torch.float32, "w"), _ptr(row_scale, torch.float32, "row_scale"),
        _ptr(col_scale, torch.float32, "col_scale"), C.c_int64(n_rows),
        _ptr(X, torch.float32, "X"), C.c_int64(ld_x), C.c_int32(d),
        _ptr(Y, torch.float32, "Y"), C.c_int64(ld_y), _ptr(addend, torch.float32, "addend"),
        C.c_int64(ld_addend), C.c_int64(addend_rows), _ptr(row_order, torch.int32, "row_order"),
        C.c_int32(chunk),
        _ptr(long_rows, torch.int32, "long_rows"), _ptr(long_ptr, torch.int64, "long_ptr"),
        C.c_int64(n_long), C.c_int64(n_tasks), _stream()))


def sylvie_aggregate_csr_fwd_wire(rowptr, col, w, row_scale, col_scale, n_rows, X, ld_x, d, n_dense,
                                  wire, n_wire, Y, ld_y, chunk=0, long_rows=None,
                                  long_ptr=None, n_long=0, n_tasks=0, workspace=None, ld_wire=0,
                                  row_order=None, bits=1):
    """bits = 1: sylvie_aggregate_csr_fwd_wire; 2, 4, 8: sylvie_aggregate_csr_fwd_wire_bbit."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = lib().sylvie_aggregate_csr_fwd_wire if bits == 1 else lib().sylvie_aggregate_csr_fwd_wire_bbit
    extra = [] if bits == 1 else [C.c_int32(bits)]
    _check(fn(
        _ptr(rowptr, torch.int64, "rowptr"), _ptr(col, torch.int32, "col"),
        _ptr(w, torch.float32, "w"), _ptr(row_scale, torch.float32, "row_scale"),
        _ptr(col_scale, torch.float32, "col_scale"), C.c_int64(n_rows),
        _ptr(X, torch.float32, "X"), C.c_int64(ld_x), C.c_int32(d), *extra, C.c_int64(n_dense),
        _ptr(wire, torch.int64, "wire"), C.c_int64(ld_wire), C.c_int64(n_wire),
        _ptr(Y, torch.float32, "Y"),
        C.c_int64(ld_y), _ptr(row_order, torch.int32, "row_order"), C.c_int32(chunk),
        _ptr(long_rows, torch.int32, "long_rows"),
        _ptr(long_ptr, torch.int64, "long_ptr"), C.c_int64(n_long), C.c_int64(n_tasks),
        _ptr(workspace, torch.float32, "workspace"), C.c_size_t(ws_bytes), _stream()))


def sylvie_aggregate_csr_bwd(rowptrT, colT, wT, row_scale, col_scale, n_rowsT, dY, ld_dy, d, dX,
                             ld_dx, addend=None, ld_addend=0, addend_rows=0, chunk=0,
                             long_rows=None, long_ptr=None, n_long=0, n_tasks=0, workspace=None,
                             row_order=None):
    _aggregate(lib().sylvie_aggregate_csr_bwd, rowptrT, colT, wT, row_scale, col_scale, n_rowsT,
               dY, ld_dy, d, dX, ld_dx, addend, ld_addend, addend_rows, chunk, long_rows,
               long_ptr, n_long, n_tasks, workspace, row_order)


def sylvie_aggregate_csr_bwd_quantize(rowptrT, colT, wT, row_scale, col_scale, row_begin, n_rows, dY,
                                      ld_dy, d, seed, stream_id, wire_out, chunk=0, long_rows=None,
                                      long_ptr=None, n_long=0, n_tasks=0, workspace=None, ld_wire=0,
                                      row_order=None, bits=1):
    """bits = 1: sylvie_aggregate_csr_bwd_quantize; 2, 4, 8: sylvie_aggregate_csr_bwd_quantize_bbit."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = lib().sylvie_aggregate_csr_bwd_quantize if bits == 1 else lib().sylvie_aggregate_csr_bwd_quantize_bbit
    extra = [] if bits == 1 else [C.c_int32(bits)]
    _check(fn(
        _ptr(rowptrT, torch.int64, "rowptrT"), _ptr(colT, torch.int32, "colT"),
        _ptr(wT, torch.float32, "wT"), _ptr(row_scale, torch.float32, "row_scale"),
        _ptr(col_scale, torch.float32, "col_scale"), C.c_int64(row_begin), C.c_int64(n_rows),
        _ptr(dY, torch.float32, "dY"), C.c_int64(ld_dy), C.c_int32(d), *extra,
        C.c_uint64(seed & (2**64 - 1)), C.c_uint32(stream_id & 0xFFFFFFFF),
        _ptr(wire_out, torch.int64, "wire_out"), C.c_int64(ld_wire),
        _ptr(row_order, torch.int32, "row_order"), C.c_int32(chunk),
        _ptr(long_rows, torch.int32, "long_rows"), _ptr(long_ptr, torch.int64, "long_ptr"),
        C.c_int64(n_long), C.c_int64(n_tasks), _ptr(workspace, torch.float32, "workspace"),
        C.c_size_t(ws_bytes), _stream()))


def sylvie_aggregate_csr_bwd_integrate(rowptrT, colT, wT, row_scale, col_scale, row_begin, n_rows,
                                       dY, ld_dy, d, dX, ld_dx, addend, ld_addend, addend_rows,
                                       wire, n_wire, seg_ptr, seg_rows, chunk=0, long_rows=None,
                                       long_ptr=None, n_long=0, n_tasks=0, workspace=None, ld_wire=0,
                                       row_order=None, bits=1):
    """bits = 1: sylvie_aggregate_csr_bwd_integrate; 2, 4, 8: sylvie_aggregate_csr_bwd_integrate_bbit."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    fn = lib().sylvie_aggregate_csr_bwd_integrate if bits == 1 else lib().sylvie_aggregate_csr_bwd_integrate_bbit
    extra = [] if bits == 1 else [C.c_int32(bits)]
    _check(fn(
        _ptr(rowptrT, torch.int64, "rowptrT"), _ptr(colT, torch.int32, "colT"),
        _ptr(wT, torch.float32, "wT"), _ptr(row_scale, torch.float32, "row_scale"),
        _ptr(col_scale, torch.float32, "col_scale"), C.c_int64(row_begin), C.c_int64(n_rows),
        _ptr(dY, torch.float32, "dY"), C.c_int64(ld_dy), C.c_int32(d), *extra,
        _ptr(dX, torch.float32, "dX"), C.c_int64(ld_dx), _ptr(addend, torch.float32, "addend"),
        C.c_int64(ld_addend), C.c_int64(addend_rows), _ptr(wire, torch.int64, "wire"),
        C.c_int64(ld_wire), C.c_int64(n_wire), _ptr(seg_ptr, torch.int64, "seg_ptr"),
        _ptr(seg_rows, torch.int32, "seg_rows"), _ptr(row_order, torch.int32, "row_order"),
        C.c_int32(chunk),
        _ptr(long_rows, torch.int32, "long_rows"), _ptr(long_ptr, torch.int64, "long_ptr"),
        C.c_int64(n_long), C.c_int64(n_tasks), _ptr(workspace, torch.float32, "workspace"),
        C.c_size_t(ws_bytes), _stream()))


def sylvie_aggregate_csr_fwd_wire_bbit(rowptr, col, w, row_scale, col_scale, n_rows, X, ld_x, d, bits, n_dense,
                                       wire, n_wire, Y, ld_y, **kw):
    sylvie_aggregate_csr_fwd_wire(rowptr, col, w, row_scale, col_scale, n_rows, X, ld_x, d, n_dense, wire,
                                  n_wire, Y, ld_y, bits=bits, **kw)


def sylvie_aggregate_csr_bwd_quantize_bbit(rowptrT, colT, wT, row_scale, col_scale, row_begin, n_rows, dY,
                                           ld_dy, d, bits, seed, stream_id, wire_out, **kw):
    sylvie_aggregate_csr_bwd_quantize(rowptrT, colT, wT, row_scale, col_scale, row_begin, n_rows, dY, ld_dy,
                                      d, seed, stream_id, wire_out, bits=bits, **kw)


def sylvie_aggregate_csr_bwd_integrate_bbit(rowptrT, colT, wT, row_scale, col_scale, row_begin, n_rows, dY,
                                            ld_dy, d, bits, dX, ld_dx, addend, ld_addend, addend_rows, wire,
                                            n_wire, seg_ptr, seg_rows, **kw):
    sylvie_aggregate_csr_bwd_integrate(rowptrT, colT, wT, row_scale, col_scale, row_begin, n_rows, dY, ld_dy,
                                       d, dX, ld_dx, addend, ld_addend, addend_rows, wire, n_wire, seg_ptr,
                                       seg_rows, bits=bits, **kw)


def sylvie_transform_fwd(A1, ld_a1, k1, A2, ld_a2, k2, W, h, n, relu, H, ld_h):
    _check(lib().sylvie_transform_fwd(
        _ptr(A1, torch.float32, "A1"), C.c_int64(ld_a1), C.c_int32(k1),
        _ptr(A2, torch.float32, "A2"), C.c_int64(ld_a2), C.c_int32(k2),
        _ptr(W, torch.float32, "W"), C.c_int32(h), C.c_int64(n), C.c_int32(int(relu)),
        _ptr(H, torch.float32, "H"), C.c_int64(ld_h), _stream()))


def sylvie_transform_bwd_workspace_bytes(k1, k2, h, n) -> int:
    return int(lib().sylvie_transform_bwd_workspace_bytes(int(k1), int(k2), int(h), int(n)))


def sylvie_transform_bwd(A1, ld_a1, k1, A2, ld_a2, k2, W, h, n, relu, H, ld_h, J, ld_j, G, dA1,
                         ld_da1, dA2, ld_da2, workspace):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sylvie_transform_bwd(
        _ptr(A1, torch.float32, "A1"), C.c_int64(ld_a1), C.c_int32(k1),
        _ptr(A2, torch.float32, "A2"), C.c_int64(ld_a2), C.c_int32(k2),
        _ptr(W, torch.float32, "W"), C.c_int32(h), C.c_int64(n), C.c_int32(int(relu)),
        _ptr(H, torch.float32, "H"), C.c_int64(ld_h), _ptr(J, torch.float32, "J"),
        C.c_int64(ld_j), _ptr(G, torch.float32, "G"), _ptr(dA1, torch.float32, "dA1"),
        C.c_int64(ld_da1), _ptr(dA2, torch.float32, "dA2"), C.c_int64(ld_da2),
        _ptr(workspace, torch.float32, "workspace"), C.c_size_t(ws_bytes), _stream()))


def sylvie_softmax_xent(H, ld_h, n, n_classes, label, count, J, ld_j, loss_rows, loss_out):
    _check(lib().sylvie_softmax_xent(
        _ptr(H, torch.float32, "H"), C.c_int64(ld_h), C.c_int64(n), C.c_int32(n_classes),
        _ptr(label, torch.int32, "label"), C.c_double(float(count)), _ptr(J, torch.float32, "J"),
        C.c_int64(ld_j), _ptr(loss_rows, torch.float32, "loss_rows"),
        _ptr(loss_out, torch.float64, "loss_out"), _stream()))


def sylvie_sum_gradients(dst, srcs, n_src, elems):
    """srcs: list of n_src float32 GPU tensors."""
    ptrs = (C.c_void_p * n_src)(*[_ptr(t, torch.float32, "src").value for t in srcs[:n_src]])
    _check(lib().sylvie_sum_gradients(_ptr(dst, torch.float32, "dst"), ptrs, C.c_int32(n_src),
                                      C.c_int64(elems), _stream()))


def sylvie_sgd_update(W, G, elems, eta):
    _check(lib().sylvie_sgd_update(_ptr(W, torch.float32, "W"), _ptr(G, torch.float32, "G"),
                                   C.c_int64(elems), C.c_float(eta), _stream()))


# ---- attention aggregator ------------------------------------------------------------------
# `pieces` is the tuple (piece_ptr int64, piece_row int32, row_piece int64) of graph_engine.piece_table.

def _pieces(pieces):
    pp, pr, rp = pieces
    return (_ptr(pp, torch.int64, "piece_ptr"), _ptr(pr, torch.int32, "piece_row"),
            _ptr(rp, torch.int64, "row_piece"), C.c_int64(pr.numel()), C.c_int64(rp.numel() - 1))


def _ws(workspace):
    n = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return _ptr(workspace, None, "workspace"), C.c_size_t(n)


def sylvie_row_dot(P, ld_p, n, F, a, out):
    _check(lib().sylvie_row_dot(_ptr(P, torch.float32, "P"), C.c_int64(ld_p), C.c_int64(n), C.c_int32(F),
                                _ptr(a, torch.float32, "a"), _ptr(out, torch.float32, "out"), _stream()))


def sylvie_edge_softmax_workspace_bytes(n_pieces, n_rows) -> int:
    return int(lib().sylvie_edge_softmax_workspace_bytes(int(n_pieces), int(n_rows)))


def sylvie_edge_softmax_fwd(pieces, col, s_dst, s_src, slope, alpha, workspace):
    _check(lib().sylvie_edge_softmax_fwd(
        *_pieces(pieces), _ptr(col, torch.int32, "col"), _ptr(s_dst, torch.float32, "s_dst"),
        _ptr(s_src, torch.float32, "s_src"), C.c_float(slope), _ptr(alpha, torch.float32, "alpha"),
        *_ws(workspace), _stream()))


def sylvie_sddmm(pieces, col, A, ld_a, Bm, ld_b, F, out):
    _check(lib().sylvie_sddmm(
        *_pieces(pieces), _ptr(col, torch.int32, "col"), _ptr(A, torch.float32, "A"), C.c_int64(ld_a),
        _ptr(Bm, torch.float32, "B"), C.c_int64(ld_b), C.c_int32(F), _ptr(out, torch.float32, "out"),
        _stream()))


def sylvie_edge_softmax_bwd(pieces, col, alpha, dalpha, s_dst, s_src, slope, de, workspace):
    _check(lib().sylvie_edge_softmax_bwd(
        *_pieces(pieces), _ptr(col, torch.int32, "col"), _ptr(alpha, torch.float32, "alpha"),
        _ptr(dalpha, torch.float32, "dalpha"), _ptr(s_dst, torch.float32, "s_dst"),
        _ptr(s_src, torch.float32, "s_src"), C.c_float(slope), _ptr(de, torch.float32, "de"),
        *_ws(workspace), _stream()))


def sylvie_segment_sum(pieces, vals, out, workspace):
    _check(lib().sylvie_segment_sum(*_pieces(pieces), _ptr(vals, torch.float32, "vals"),
                                    _ptr(out, torch.float32, "out"), *_ws(workspace), _stream()))


def sylvie_permute_f32(inp, perm, n, out):
    _check(lib().sylvie_permute_f32(_ptr(inp, torch.float32, "in"), _ptr(perm, torch.int64, "perm"),
                                    C.c_int64(n), _ptr(out, torch.float32, "out"), _stream()))


def sylvie_rank1_add(X, ld_x, n, F, s, a):
    _check(lib().sylvie_rank1_add(_ptr(X, torch.float32, "X"), C.c_int64(ld_x), C.c_int64(n), C.c_int32(F),
                                  _ptr(s, torch.float32, "s"), _ptr(a, torch.float32, "a"), _stream()))


def sylvie_relu_fwd(Z, ld_z, n, F, H, ld_h):
    _check(lib().sylvie_relu_fwd(_ptr(Z, torch.float32, "Z"), C.c_int64(ld_z), C.c_int64(n), C.c_int32(F),
                                 _ptr(H, torch.float32, "H"), C.c_int64(ld_h), _stream()))


def sylvie_relu_bwd(H, ld_h, J, ld_j, n, F, dZ, ld_dz):
    _check(lib().sylvie_relu_bwd(_ptr(H, torch.float32, "H"), C.c_int64(ld_h), _ptr(J, torch.float32, "J"),
                                 C.c_int64(ld_j), C.c_int64(n), C.c_int32(F), _ptr(dZ, torch.float32, "dZ"),
                                 C.c_int64(ld_dz), _stream()))


def sylvie_scaled_column_sum_workspace_bytes(n, F) -> int:
    return int(lib().sylvie_scaled_column_sum_workspace_bytes(int(n), int(F)))


def sylvie_scaled_column_sum(X, ld_x, n, F, s, out, workspace):
    _check(lib().sylvie_scaled_column_sum(_ptr(X, torch.float32, "X"), C.c_int64(ld_x), C.c_int64(n),
                                          C.c_int32(F), _ptr(s, torch.float32, "s"),
                                          _ptr(out, torch.float32, "out"), *_ws(workspace), _stream()))


# ---- the attention aggregator for K heads at once ([.][K] arrays) -------------------------

def sylvie_row_dot_heads(P, ld_p, n, F, heads, a, out, a2=None, n2=0, out2=None):
    _check(lib().sylvie_row_dot_heads(_ptr(P, torch.float32, "P"), C.c_int64(ld_p), C.c_int64(n), C.c_int32(F),
                                      C.c_int32(heads), _ptr(a, torch.float32, "a"),
                                      _ptr(out, torch.float32, "out"), _ptr(a2, torch.float32, "a2"),
                                      C.c_int64(n2), _ptr(out2, torch.float32, "out2"), _stream()))


def sylvie_edge_softmax_heads_workspace_bytes(n_pieces, n_rows, heads) -> int:
    return int(lib().sylvie_edge_softmax_heads_workspace_bytes(int(n_pieces), int(n_rows), int(heads)))


def sylvie_edge_softmax_fwd_heads(pieces, col, s_dst, s_src, heads, slope, alpha, workspace):
    _check(lib().sylvie_edge_softmax_fwd_heads(
        *_pieces(pieces), _ptr(col, torch.int32, "col"), _ptr(s_dst, torch.float32, "s_dst"),
        _ptr(s_src, torch.float32, "s_src"), C.c_int32(heads), C.c_float(slope),
        _ptr(alpha, torch.float32, "alpha"), *_ws(workspace), _stream()))


def sylvie_sddmm_heads(pieces, col, A, ld_a, Bm, ld_b, F, heads, out):
    _check(lib().sylvie_sddmm_heads(
        *_pieces(pieces), _ptr(col, torch.int32, "col"), _ptr(A, torch.float32, "A"), C.c_int64(ld_a),
        _ptr(Bm, torch.float32, "B"), C.c_int64(ld_b), C.c_int32(F), C.c_int32(heads),
        _ptr(out, torch.float32, "out"), _stream()))


def sylvie_edge_softmax_bwd_heads(pieces, col, alpha, dalpha, s_dst, s_src, heads, slope, de, ds_dst,
                                  workspace):
    _check(lib().sylvie_edge_softmax_bwd_heads(
        *_pieces(pieces), _ptr(col, torch.int32, "col"), _ptr(alpha, torch.float32, "alpha"),
        _ptr(dalpha, torch.float32, "dalpha"), _ptr(s_dst, torch.float32, "s_dst"),
        _ptr(s_src, torch.float32, "s_src"), C.c_int32(heads), C.c_float(slope),
        _ptr(de, torch.float32, "de"), _ptr(ds_dst, torch.float32, "ds_dst"), *_ws(workspace), _stream()))


def sylvie_segment_sum_heads(pieces, vals, index, heads, out, workspace):
    _check(lib().sylvie_segment_sum_heads(
        *_pieces(pieces), _ptr(vals, torch.float32, "vals"), _ptr(index, torch.int64, "index"),
        C.c_int32(heads), _ptr(out, torch.float32, "out"), *_ws(workspace), _stream()))


def sylvie_scaled_column_sum_heads(X, ld_x, n, F, heads, s, out, workspace, s2=None, n2=0, out2=None):
    _check(lib().sylvie_scaled_column_sum_heads(
        _ptr(X, torch.float32, "X"), C.c_int64(ld_x), C.c_int64(n), C.c_int32(F), C.c_int32(heads),
        _ptr(s, torch.float32, "s"), _ptr(out, torch.float32, "out"), _ptr(s2, torch.float32, "s2"),
        C.c_int64(n2), _ptr(out2, torch.float32, "out2"), *_ws(workspace), _stream()))


def sylvie_aggregate_csr_attention(rowptr, col, w, w_index, heads, n_rows, X, ld_x, d, Y, ld_y, s1=None,
                                   a1=None, n1=0, s2=None, a2=None, n2=0, relu=False, chunk=0,
                                   long_rows=None, long_ptr=None, n_long=0, n_tasks=0, workspace=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sylvie_aggregate_csr_attention(
        _ptr(rowptr, torch.int64, "rowptr"), _ptr(col, torch.int32, "col"), _ptr(w, torch.float32, "w"),
        _ptr(w_index, torch.int64, "w_index"), C.c_int32(heads), C.c_int64(n_rows),
        _ptr(X, torch.float32, "X"), C.c_int64(ld_x), C.c_int32(d), _ptr(Y, torch.float32, "Y"),
        C.c_int64(ld_y), _ptr(s1, torch.float32, "s1"), _ptr(a1, torch.float32, "a1"), C.c_int64(n1),
        _ptr(s2, torch.float32, "s2"), _ptr(a2, torch.float32, "a2"), C.c_int64(n2), C.c_int32(int(relu)),
        C.c_int32(chunk), _ptr(long_rows, torch.int32, "long_rows"), _ptr(long_ptr, torch.int64, "long_ptr"),
        C.c_int64(n_long), C.c_int64(n_tasks), _ptr(workspace, torch.float32, "workspace"),
        C.c_size_t(ws_bytes), _stream()))


def sylvie_seed_offset_source(offset):
    """offset: a one-element int64 GPU tensor (kept alive by the caller) or None."""
    _check(lib().sylvie_seed_offset_source(_ptr(offset, torch.int64, "offset")))


def sylvie_rank1_add_heads(X, ld_x, F, heads, s1, a1, n1, s2=None, a2=None, n2=0):
    _check(lib().sylvie_rank1_add_heads(
        _ptr(X, torch.float32, "X"), C.c_int64(ld_x), C.c_int32(F), C.c_int32(heads),
        _ptr(s1, torch.float32, "s1"), _ptr(a1, torch.float32, "a1"), C.c_int64(n1),
        _ptr(s2, torch.float32, "s2"), _ptr(a2, torch.float32, "a2"), C.c_int64(n2), _stream()))


def sylvie_aggregate_csr_attention_sddmm_supported(d, heads) -> bool:
    return bool(lib().sylvie_aggregate_csr_attention_sddmm_supported(C.c_int32(d), C.c_int32(heads)))


def sylvie_aggregate_csr_attention_sddmm(rowptr, col, w, w_index, heads, n_rows, X, ld_x, d, Y, ld_y, Bm, ld_b,
                                         dalpha, chunk=0, long_rows=None, long_ptr=None, n_long=0, n_tasks=0,
                                         workspace=None):
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().sylvie_aggregate_csr_attention_sddmm(
        _ptr(rowptr, torch.int64, "rowptr"), _ptr(col, torch.int32, "col"), _ptr(w, torch.float32, "w"),
        _ptr(w_index, torch.int64, "w_index"), C.c_int32(heads), C.c_int64(n_rows),
        _ptr(X, torch.float32, "X"), C.c_int64(ld_x), C.c_int32(d), _ptr(Y, torch.float32, "Y"),
        C.c_int64(ld_y), _ptr(Bm, torch.float32, "B"), C.c_int64(ld_b), _ptr(dalpha, torch.float32, "dalpha"),
        C.c_int32(chunk), _ptr(long_rows, torch.int32, "long_rows"), _ptr(long_ptr, torch.int64, "long_ptr"),
        C.c_int64(n_long), C.c_int64(n_tasks), _ptr(workspace, torch.float32, "workspace"),
        C.c_size_t(ws_bytes), _stream()))


# ---- Graph Engine set-up (each call waits for the current stream) ------------------------

def sylvie_graph_workspace_bytes(n) -> int:
    return int(lib().sylvie_graph_workspace_bytes(int(n)))


def sylvie_graph_local_index(gcol, nnz, n_in, owner, n_nodes, part, pos, halo_gid, halo_capacity, workspace):
    """Returns (|V_n|, |V_HALO,n|) as the library reported them; raises on a failed check."""
    counts = (C.c_int64 * 2)(0, 0)
    _check(lib().sylvie_graph_local_index(_ptr(gcol, torch.int32, "gcol"), C.c_int64(nnz), C.c_int64(n_in),
                                          _ptr(owner, torch.int32, "owner"), C.c_int64(n_nodes), C.c_int32(part),
                                          _ptr(pos, torch.int32, "pos"), _ptr(halo_gid, torch.int32, "halo_gid"),
                                          C.c_int64(halo_capacity), counts, *_ws(workspace), _stream()))
    return int(counts[0]), int(counts[1])


def sylvie_graph_relabel_columns(gcol, nnz, pos, n_nodes, col, workspace):
    _check(lib().sylvie_graph_relabel_columns(_ptr(gcol, torch.int32, "gcol"), C.c_int64(nnz),
                                              _ptr(pos, torch.int32, "pos"), C.c_int64(n_nodes),
                                              _ptr(col, torch.int32, "col"), *_ws(workspace), _stream()))


def sylvie_graph_rows_in_owner(owner, n_nodes, n_parts, row_of, part_ptr, workspace):
    _check(lib().sylvie_graph_rows_in_owner(_ptr(owner, torch.int32, "owner"), C.c_int64(n_nodes), C.c_int32(n_parts),
                                            _ptr(row_of, torch.int32, "row_of"), _ptr(part_ptr, torch.int64, "part_ptr"),
                                            *_ws(workspace), _stream()))


def sylvie_graph_recv_sets(halo_gid, n_halo, owner, row_of, n_nodes, n_parts, R_ptr, R_halo, R_row, workspace):
    _check(lib().sylvie_graph_recv_sets(_ptr(halo_gid, torch.int32, "halo_gid"), C.c_int64(n_halo),
                                        _ptr(owner, torch.int32, "owner"), _ptr(row_of, torch.int32, "row_of"),
                                        C.c_int64(n_nodes), C.c_int32(n_parts), _ptr(R_ptr, torch.int64, "R_ptr"),
                                        _ptr(R_halo, torch.int32, "R_halo"), _ptr(R_row, torch.int32, "R_row"),
                                        *_ws(workspace), _stream()))


def sylvie_graph_transpose_csr(rowptr, col, w, n_rows, n_cols, nnz, rowptrT, colT, wT, perm, workspace):
    _check(lib().sylvie_graph_transpose_csr(_ptr(rowptr, torch.int64, "rowptr"), _ptr(col, torch.int32, "col"),
                                            _ptr(w, torch.float32, "w"), C.c_int64(n_rows), C.c_int64(n_cols),
                                            C.c_int64(nnz), _ptr(rowptrT, torch.int64, "rowptrT"),
                                            _ptr(colT, torch.int32, "colT"), _ptr(wT, torch.float32, "wT"),
                                            _ptr(perm, torch.int64, "perm"), *_ws(workspace), _stream()))


def sylvie_graph_scatter_segments(dst_row, n, n_dst, seg_ptr, seg_rows, workspace):
    _check(lib().sylvie_graph_scatter_segments(_ptr(dst_row, torch.int32, "dst_row"), C.c_int64(n), C.c_int64(n_dst),
                                               _ptr(seg_ptr, torch.int64, "seg_ptr"),
                                               _ptr(seg_rows, torch.int32, "seg_rows"), *_ws(workspace), _stream()))


def sylvie_graph_gcn_operator(rowptr, col, deg, n_in, n_cols, nnz, rowptr_out, col_out, w_out, workspace):
    _check(lib().sylvie_graph_gcn_operator(_ptr(rowptr, torch.int64, "rowptr"), _ptr(col, torch.int32, "col"),
                                           _ptr(deg, torch.int32, "deg"), C.c_int64(n_in), C.c_int64(n_cols),
                                           C.c_int64(nnz), _ptr(rowptr_out, torch.int64, "rowptr_out"),
                                           _ptr(col_out, torch.int32, "col_out"), _ptr(w_out, torch.float32, "w_out"),
                                           *_ws(workspace), _stream()))


def sylvie_graph_mean_weights(rowptr, n_rows, nnz, w_out, workspace):
    _check(lib().sylvie_graph_mean_weights(_ptr(rowptr, torch.int64, "rowptr"), C.c_int64(n_rows), C.c_int64(nnz),
                                           _ptr(w_out, torch.float32, "w_out"), *_ws(workspace), _stream()))


def sylvie_graph_long_row_plan(rowptr, row_begin, n_rows, chunk, long_rows, long_ptr, capacity, workspace):
    """Returns (n_long, n_tasks) as the library reported them."""
    counts = (C.c_int64 * 2)(0, 0)
    _check(lib().sylvie_graph_long_row_plan(_ptr(rowptr, torch.int64, "rowptr"), C.c_int64(row_begin), C.c_int64(n_rows),
                                            C.c_int32(chunk), _ptr(long_rows, torch.int32, "long_rows"),
                                            _ptr(long_ptr, torch.int64, "long_ptr"), C.c_int64(capacity), counts,
                                            *_ws(workspace), _stream()))
    return int(counts[0]), int(counts[1])


def sylvie_graph_piece_table(rowptr, n_rows, chunk, row_piece, piece_ptr, piece_row, capacity, workspace):
    """Returns the number of pieces."""
    count = (C.c_int64 * 1)(0)
    _check(lib().sylvie_graph_piece_table(_ptr(rowptr, torch.int64, "rowptr"), C.c_int64(n_rows), C.c_int32(chunk),
                                          _ptr(row_piece, torch.int64, "row_piece"), _ptr(piece_ptr, torch.int64, "piece_ptr"),
                                          _ptr(piece_row, torch.int32, "piece_row"), C.c_int64(capacity), count,
                                          *_ws(workspace), _stream()))
    return int(count[0])


def sylvie_graph_rows_by_length(rowptr, row_begin, n_rows, order, workspace):
    _check(lib().sylvie_graph_rows_by_length(_ptr(rowptr, torch.int64, "rowptr"), C.c_int64(row_begin), C.c_int64(n_rows),
                                             _ptr(order, torch.int32, "order"), *_ws(workspace), _stream()))
