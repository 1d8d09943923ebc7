"""The committed rocprofv3 summary that bench.py's roofline object reads must be a profile of the
kernel sources in the tree: it names their digest, and bench.py ignores it otherwise."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_step_profile_names_the_sources_in_the_tree():
    sys.path.insert(0, ROOT)
    import bench
    prof = bench.read_profile()
    assert prof, "profiles/stress_step_kernels.txt is of other kernel sources: profile the step again"
    for name in ("sylvie_quantize_1bit_fwd", "sylvie_aggregate_csr_fwd_wire", "sylvie_transform_fwd",
                 "sylvie_transform_bwd", "sylvie_aggregate_csr_bwd_quantize", "sylvie_aggregate_csr_bwd_integrate"):
        p = prof[name]
        assert p["kernel_ms"] > 0 and p["event_ms"] > 0 and p["fetched"] > 0 and p["written"] > 0
        # an event-bracketed call cannot be much shorter than its kernels
        assert p["event_ms"] > 0.9 * p["kernel_ms"]
