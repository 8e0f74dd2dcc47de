"""MI355X-native single-GPU memgraph runtime (taskgraph -> BuildMemgraph -> event-driven execution).

The product is libturnip.so (C ABI in include/turnip.h).  `binding` mirrors that ABI one to one
with ctypes; `harness` only marshals arrays in and out.  Every step of the method runs inside
the library; there is no Python or CPU fallback.
"""
from . import binding  # noqa: F401
