"""LCKV decode attention for MI355X (gfx950): thin Python binding over the C-ABI library ``liblckv.so``.

The binding (``paper_2405_10637_amd.binding``) only marshals arguments; every step of the decode path runs
in the HIP kernels.  Importing the package does not load the library, so the input generators in
``paper_2405_10637_amd.synth`` work on a machine without it; calling any ``lckv_*`` function without the
built library raises.
"""
