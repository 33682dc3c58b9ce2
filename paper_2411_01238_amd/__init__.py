"""libsdrop: SparseDrop's block-dropout-fused GEMMs as hand-written HIP kernels for gfx950.

``paper_2411_01238_amd.sdrop`` is the thin binding over the C-ABI library
(``include/sdrop.h``); ``paper_2411_01238_amd.workloads`` holds the seeded
synthetic inputs.  Nothing is imported eagerly so that the input generators can
be used without the HIP library.
"""
