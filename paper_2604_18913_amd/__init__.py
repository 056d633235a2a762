"""MI355X-native batched k-hop knowledge-graph retrieval (LogosKG hot path).

The work is done by ``liblogoskg.so`` (hand-written HIP for gfx950, C ABI in
``include/logoskg.h``); this package is a thin ctypes binding with the same
names.  PyTorch is used only for device buffers and the stream handle.
"""
from .binding import (Graph, Result, LogosKGError, logoskg_build, logoskg_khop, logoskg_paths,
                      library_path, version)

__all__ = ["Graph", "Result", "LogosKGError", "logoskg_build", "logoskg_khop", "logoskg_paths",
           "library_path", "version"]
