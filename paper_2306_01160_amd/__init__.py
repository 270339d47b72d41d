"""Sparse Causal Flash Attention for MI355X (gfx950): HIP kernels behind a C ABI.

``binding`` wraps ``libscfa.so`` (same function names as ``include/scfa.h``;
argument marshalling only).  ``pipeline`` chains the entry points into the two
variants' forward / backward passes.  ``workloads`` draws the seeded synthetic
inputs.  Importing this package does not load the library; the first call does,
and it raises if the library has not been built (``python -m paper_2306_01160_amd.build``).
"""
__all__ = ["binding", "pipeline", "workloads", "build"]
