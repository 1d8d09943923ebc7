"""Shared test helpers: turn synthetic workloads into the oracle's plain arrays."""
import numpy as np

from oracle.layers import PartData


def np_c(t, dtype=None):
    a = t.detach().cpu().numpy()
    if dtype is not None:
        a = a.astype(dtype, copy=False)
    return np.ascontiguousarray(a)


def to_partdata(wl, loopback=None):
    """synth.Workload -> [PartData].  With a loopback mirror every halo row is owned by
    partition 0 itself at inner row mirror[j]."""
    out = []
    for i, p in enumerate(wl.parts):
        if wl.mirror is not None:
            hp = np.zeros(p.n_halo, np.int32)
            hr = np_c(wl.mirror, np.int32)
        else:
            hp = np_c(p.halo_part, np.int32)
            hr = np_c(p.halo_row, np.int32)
        out.append(PartData(
            n_in=p.n_in, n_halo=p.n_halo, rowptr=np_c(p.rowptr, np.int64),
            col=np_c(p.col, np.int32), deg=np_c(p.deg, np.int32), halo_part=hp, halo_row=hr,
            X=np_c(wl.X[i], np.float32), J=np_c(wl.J[i], np.float32)))
    return out


def ulp32(x):
    x = np.abs(np.asarray(x, np.float32))
    return np.spacing(x)


def split_wire(wire, n, d):
    """GPU wire (uint64 [n][W+1], as an int64/uint64 array) -> the oracle's three arrays:
    packed uint64 [n, W], scale f32 [n], zero f32 [n]."""
    W = (d + 63) // 64
    w = np.ascontiguousarray(wire).view(np.uint64)[: n * (W + 1)].reshape(n, W + 1)
    meta = np.ascontiguousarray(w[:, W])
    scale = (meta & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.float32)
    zero = (meta >> np.uint64(32)).astype(np.uint32).view(np.float32)
    return np.ascontiguousarray(w[:, :W]), scale, zero


def join_wire(packed, scale, zero):
    """The oracle's three arrays -> wire rows uint64 [n][W+1] (returned as int64 for torch)."""
    n, W = packed.shape
    w = np.empty((n, W + 1), np.uint64)
    w[:, :W] = packed
    w[:, W] = (zero.view(np.uint32).astype(np.uint64) << np.uint64(32)) | \
        scale.view(np.uint32).astype(np.uint64)
    return w.view(np.int64)
