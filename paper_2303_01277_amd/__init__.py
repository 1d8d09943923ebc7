"""MI355X (gfx950) hot path of Sylvie's 1-bit boundary exchange on one graph partition.

`binding` holds thin ctypes wrappers, one per entry point of include/sylvie.h (same
names, argument marshalling only); `graph_engine` the one-off host-side set-up
(normalised operators, transposed CSR, long-row plans, scatter segments);
`trainer` the per-layer call sequence of Alg. 1 / Alg. 2.  Nothing here computes
on the CPU: without the built HIP library every call raises.
"""
from .build import build_library, library_path  # noqa: F401
