"""NestedFP hot path for MI355X (gfx950): byte-plane decompose / reconstruct and
the dual-mode linear-layer GEMM, as a C-ABI HIP library plus this thin binding.

Importing the package does not load the HIP library; the first call into
``paper_2506_02024_amd.binding`` does, and fails loudly if it is not built.
"""
__all__ = ["binding", "workloads", "build"]
