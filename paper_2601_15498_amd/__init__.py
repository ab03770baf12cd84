"""MARS margin-aware speculative verification for AMD MI355X (gfx950).

The package is a thin binding over the C-ABI library ``libmars.so`` (HIP kernels in
``csrc/``).  PyTorch is used for device memory and streams only; every step of the
verification pass runs in the library's kernels.  There is no CPU fallback: importing
:mod:`paper_2601_15498_amd.binding` without the built library raises.
"""
__all__ = ["binding", "build"]
