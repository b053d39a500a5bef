"""Light Forcing's per-chunk Hierarchical Sparse Attention for AMD MI355X (gfx950).

``paper_2602_04789_amd.lf``    -- ctypes binding of the C-ABI library (HIP kernels).
``paper_2602_04789_amd.synth`` -- seeded synthetic inputs (numpy only).
``paper_2602_04789_amd.build`` -- compiles the library with hipcc for gfx950.

Importing the package loads nothing; the binding loads the shared library on first
use and raises if it has not been built.
"""
__all__ = ["lf", "synth", "build"]
