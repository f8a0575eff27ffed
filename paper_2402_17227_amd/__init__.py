"""MI355X-native sampled linear-layer backward of VCAS (arxiv 2402.17227).

The work is done by hand-written gfx950 kernels in ``libvcas.so`` (C ABI in
``include/vcas.h``); :mod:`paper_2402_17227_amd.binding` is a thin ctypes layer
with the same names.  Importing this package does not load the library."""

__all__ = ["binding", "build"]
