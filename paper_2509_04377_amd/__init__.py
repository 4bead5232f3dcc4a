"""PagedEviction hot path for AMD MI355X (gfx950): hand-written HIP kernels behind a C ABI.

`binding` marshals torch tensors into the C-ABI calls of libpe.so (include/pe.h); `synth` draws
the seeded synthetic workloads.  Nothing here computes on the CPU: if libpe.so has not been built
the first call raises.
"""
from . import synth  # noqa: F401

__all__ = ["synth", "binding", "build"]
