"""MI355X-native batch-1 decoder inference (libedgefm) -- Python side.

The product is the C-ABI shared library built from ``csrc/`` (declared in
``include/edgefm.h``); :mod:`.binding` is a thin ctypes layer with the same
entry-point names.  Importing this package does not load the library.
"""
from .buildlib import build, lib_path  # noqa: F401
