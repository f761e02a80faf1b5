"""libdhelix: Strand-Interleaving layer step for MI355X (gfx950).

`paper_2411_15871_amd.dhelix` is the ctypes binding of the C-ABI library (it raises if the
HIP library has not been built); `paper_2411_15871_amd.inputs` draws the seeded synthetic
inputs.  Nothing is imported eagerly so the input generator can be used without the library.
"""
