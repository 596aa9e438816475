"""MI355X-native sparse 3D-attention forward of Sparse-vDiT (arxiv 2506.03065).

`paper_2506_03065_amd.binding` wraps the C-ABI library (HIP kernels for gfx950 +
host pattern compiler); `paper_2506_03065_amd.workloads` draws seeded synthetic
inputs.  Importing the package does not load the shared library; the binding
does, and fails loudly when it is missing.
"""
__all__ = ["binding", "workloads"]
