"""MI355X-native batched decode attention over a paged KV cache (gfx950 HIP kernels behind a C ABI).

Importing the package loads nothing native: `paper_2602_02204_amd.binding` opens the
HIP library on first use and raises if it has not been built.
"""
__all__ = ["binding", "workloads"]
