"""MI355X-native residual-CNN training hot path (conv fwd/dgrad/wgrad + fused BN/ReLU/add).

`binding` is the ctypes front end of libnsk.so (the C ABI of include/nsk.h); `network` issues the
call sequence of a whole residual workload through it.  Build the library with
``python -m paper_2409_11600_amd.build``.
"""
from . import binding  # noqa: F401
