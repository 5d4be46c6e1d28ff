"""xKV Selective-Reconstruction decode attention for AMD MI355X (gfx950).

`binding` exposes the C ABI of libxkv (include/xkv.h); `synth` holds the seeded synthetic
workloads; `build` compiles the HIP sources in-tree.
"""
from . import binding, synth  # noqa: F401
from .binding import Shape  # noqa: F401

__all__ = ["binding", "synth", "Shape"]
