"""MI355X-native Transformer encoder layer (forward + backward) behind a C ABI.

The product is ``libflmi355.so`` (built by ``paper_2201_12465_amd.build``) and its
header ``include/fl_layer.h``; ``binding`` is the ctypes wrapper with the same names.
"""
from . import binding  # noqa: F401
