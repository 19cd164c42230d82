"""MI355X-native exact attention (forward and backward), hand-written HIP for gfx950.

`paper_2307_08691_amd.binding` is the thin ctypes layer over the C ABI declared
in include/fa.h; `paper_2307_08691_amd.inputs` draws the seeded synthetic
workloads. Importing the package loads neither torch nor the shared library.
"""
__all__ = ["binding", "inputs", "build"]
