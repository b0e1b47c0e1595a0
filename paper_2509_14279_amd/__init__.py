"""Fused dense-layer block (Linear -> GELU_erf -> LayerNorm, forward and full
backward) for AMD MI355X: hand-written HIP kernels behind a C-ABI library,
with a thin ctypes binding.  Importing the package does not load the library;
`paper_2509_14279_amd.api` does, and fails loudly when it is missing."""

__all__ = ["inputs"]
