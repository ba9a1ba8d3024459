"""MI355X-native ResQ mixed-precision (INT8 + INT4) quantized linear layer.

The compute lives in hand-written gfx950 HIP kernels behind a C ABI
(``include/resq.h``); :mod:`paper_2412_14363_amd.binding` marshals arguments
to it.  Nothing is imported eagerly so that the input generators can be used
without the HIP library.
"""
__all__ = ["binding", "workloads", "build"]
