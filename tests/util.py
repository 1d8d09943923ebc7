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
