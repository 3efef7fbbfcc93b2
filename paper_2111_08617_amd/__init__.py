"""MI355X-native hot path of CGX's compressed gradient communication.

The compute lives in ``libcgx.so`` (hand-written HIP for gfx950 behind a C ABI,
see ``include/cgx.h``); :mod:`.binding` is the thin ctypes layer over it and
:mod:`.workloads` the seeded synthetic inputs.  Nothing here loads the library
at import time; the first call does, and raises if it has not been built.
"""
__all__ = ["binding", "workloads", "build"]
