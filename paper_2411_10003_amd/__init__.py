"""One GPU's share of an expert-parallel MoE layer on MI355X (gfx950).

`binding` wraps the C-ABI library (hand-written HIP kernels); `workload` draws the seeded
synthetic inputs.  Importing the package loads nothing native: `binding.load()` does, and
it raises if the library has not been built.
"""
__all__ = ["binding", "workload", "build"]
