"""MI355X-native fused forward of Diagonal-Tiled Mixed-Precision Attention (DMA).

``paper_2604_03950_amd.binding`` is the thin Python layer over the C-ABI library
(``libdma_mi355x.so``, hand-written HIP for gfx950); ``paper_2604_03950_amd.workloads`` holds the
seeded synthetic input generators.  Importing the package loads nothing; the binding loads the
shared library on first use and raises if it has not been built.
"""

__all__ = ["binding", "workloads", "build"]
