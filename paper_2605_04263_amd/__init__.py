"""Parallel prefix verification attention for AMD MI355X (gfx950).

`paper_2605_04263_amd.binding` loads the HIP library and exposes the C ABI of include/pv.h;
`paper_2605_04263_amd.build` compiles it.  Importing this package does not load the library.
"""
__all__ = ["binding", "build"]
