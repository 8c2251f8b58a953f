"""Fused chains of memory-intensive operators as single HIP kernels on MI355X (gfx950).

`binding` mirrors the C ABI declared in include/pf_chain.h.  Importing it requires the built shared
library (paper_2307_04995_amd/lib/libpf_chain.so); there is no CPU or eager fallback.
"""
from . import build as _build  # noqa: F401  (build helper; does not compile on import)

__all__ = ["binding", "build"]
