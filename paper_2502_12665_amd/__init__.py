"""MI355X (gfx950) implementation of the A2ATS decode-time retrieval path.

`binding` is the ctypes layer over the C ABI (include/a2ats.h); `synth` holds the seeded
synthetic workloads; `build` compiles the HIP library in-tree.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding", "build"]
