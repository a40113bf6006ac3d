"""MI355X-native batched MMBP local search, lower bound and online iteration simulator.

The compute path lives in ``libmmbp.so`` (hand-written HIP for gfx950, built from ``csrc/``).
``paper_2502_15763_amd.api`` is a thin argument-marshalling layer over its C ABI; importing
this package does not load the library, the first API call does (and raises if it is missing).
``paper_2502_15763_amd.workloads`` holds the seeded synthetic input generators only.
"""

__all__ = ["api", "workloads", "build"]
