"""Batched SpMM for small graphs on AMD MI355X (gfx950).

``paper_1903_11409_amd.bspmm`` is the thin binding over the C-ABI library built from ``csrc/``;
``paper_1903_11409_amd.workloads`` holds the seeded input generators.  Nothing is loaded at
import time: the shared library is opened on the first call into the binding and a missing
library is an error, never a fallback.
"""
__all__ = ["bspmm", "workloads"]
