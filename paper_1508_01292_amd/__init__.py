"""MI355X-native hot path of the compact CNN cascade detector (arXiv 1508.01292).

The work is done by hand-written HIP kernels in libcnnc.so (C ABI: include/cnnc.h).  This
package is only the ctypes binding: it marshals arguments and never computes a step itself.
"""
from . import binding as _b
from .binding import (EXPORTS, STEP_NAMES, CnncError, Context, Detection, Pipe, Records, Region, RegionDetection, Stream, lib,
                      library_path)

__all__ = ["CnncError", "Context", "Detection", "Pipe", "Records", "Region", "RegionDetection", "Stream", "lib", "library_path", "EXPORTS",
           "STEP_NAMES"]
for _n in dir(_b):
    if _n.startswith("cnnc_"):
        globals()[_n] = getattr(_b, _n)
        __all__.append(_n)
