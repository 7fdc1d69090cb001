"""fp4mr: micro-rotated FP4 (MXFP4 / NVFP4) linear-layer hot path for AMD MI355X (gfx950).

``paper_2509_23202_amd.binding`` is the thin ctypes layer over the C-ABI library ``libfp4mr.so``;
``paper_2509_23202_amd.inputs`` holds the seeded synthetic input generators.  The binding raises at
import time when the HIP library has not been built: there is no CPU fallback.
"""
__version__ = "0.1.0"
