"""Radial Attention hot path for MI355X (gfx950): block-mask builder + block-sparse attention.

``paper_2506_19852_amd.binding`` is the ctypes layer over the C-ABI library ``libradial.so``
(declared in ``include/radial.h``); ``paper_2506_19852_amd.workloads`` holds the seeded synthetic
input generators; ``paper_2506_19852_amd.build`` compiles the HIP sources in-tree.
"""
