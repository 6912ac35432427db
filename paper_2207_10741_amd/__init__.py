"""Focused convolution for MI355X (gfx950): hand-written HIP kernels behind a
C ABI, plus a thin Python binding (`paper_2207_10741_amd.binding`).

Submodules are imported on demand so that the input generators (`synth`,
`workloads`) can be used without loading the GPU library.
"""
__all__ = ["binding", "synth", "workloads"]
