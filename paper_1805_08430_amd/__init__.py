"""rdev: zero-copy tensor transfer through a memory-region "device" interface
on one MI355X (sender and receiver arenas in the same HBM).

``paper_1805_08430_amd.rdev``      ctypes binding of the C-ABI library (argument marshalling only)
``paper_1805_08430_amd.workloads`` seeded synthetic tensor sets (inputs only)
``paper_1805_08430_amd.build``     compiles csrc/ with hipcc for gfx950

Nothing is imported eagerly: the binding loads the shared library on first use
and raises if it has not been built.
"""
__all__ = ["rdev", "workloads", "build"]
