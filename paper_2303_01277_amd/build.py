"""Compile the HIP sources in csrc/ into paper_2303_01277_amd/libsylvie.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_BUILD = os.path.join(_HERE, "_build")
_SO = os.path.join(_HERE, "libsylvie.so")

_COMMON = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# per-file extras: the quantizer's float steps are single IEEE operations (no
# contraction); its inputs are finite by contract, which lets min/max be one
# instruction each.
_SOURCES = {
    "api.hip": [],
    "quantize.hip": ["-ffp-contract=off", "-fno-honor-nans"],
    "dequantize.hip": ["-ffp-contract=off"],
    "lowbit_bbit.hip": ["-ffp-contract=off", "-fno-honor-nans"],
    "aggregate.hip": ["-ffp-contract=off"],
    "transform.hip": [],
    "training.hip": ["-ffp-contract=off"],
    "gat.hip": ["-ffp-contract=off"],
    "gat_aggregate.hip": ["-ffp-contract=off"],
    "graph_engine.hip": [],
    "validate.hip": [],
}


def library_path() -> str:
    """The built library; SYLVIE_LIBRARY names another build of it (same ABI) to load instead."""
    return os.environ.get("SYLVIE_LIBRARY") or _SO


def _stale() -> bool:
    if not os.path.exists(_SO):
        return True
    t = os.path.getmtime(_SO)
    deps = [os.path.join(_CSRC, f) for f in os.listdir(_CSRC)]
    deps.append(os.path.join(os.path.dirname(_HERE), "include", "sylvie.h"))
    return any(os.path.getmtime(p) > t for p in deps)


def build_library(force: bool = False, verbose: bool = False) -> str:
    """Compile every source and link the shared library.  Returns its path."""
    if not force and not _stale():
        return _SO
    os.makedirs(_BUILD, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

    def compile_one(item):
        name, extra = item
        obj = os.path.join(_BUILD, name.replace(".hip", ".o"))
        cmd = [hipcc, *_COMMON, *extra, "-c", os.path.join(_CSRC, name), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {name}:\n{r.stdout}\n{r.stderr}")
        if verbose and r.stderr.strip():
            print(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(_SOURCES))) as ex:
        objs = list(ex.map(compile_one, _SOURCES.items()))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", _SO, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return _SO


if __name__ == "__main__":
    print(build_library(force=True, verbose=True))
