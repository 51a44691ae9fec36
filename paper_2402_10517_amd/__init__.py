"""Any-precision GEMV for MI355X (gfx950): thin Python binding over the C-ABI library.

The HIP library is loaded lazily by `paper_2402_10517_amd.binding`; importing this package
or `paper_2402_10517_amd.inputs` touches neither the GPU nor the shared library.
"""
