"""Fused transformer decoder-block forward for MI355X (gfx950).

The HIP library is loaded on first use of :mod:`paper_2604_16498_amd.binding`;
importing the package (for instance for :mod:`paper_2604_16498_amd.inputs`)
touches neither the GPU nor the shared library.
"""

__all__ = ["inputs", "binding", "build"]
