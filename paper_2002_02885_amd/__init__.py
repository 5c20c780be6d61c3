"""MI355X-native packed training (the `pack` primitive of arXiv 2002.02885).

The work is done by hand-written gfx950 kernels inside ``libpack.so`` (C ABI in ``include/pack.h``);
this package is only the ctypes binding.  Importing the package does not load the library;
the first use of :mod:`paper_2002_02885_amd.binding` does, and raises if it is missing.
"""

__all__ = ["binding", "build"]
