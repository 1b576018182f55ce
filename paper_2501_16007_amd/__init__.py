"""TopLoc proof build / verify hot path for MI355X (gfx950).

The compute lives in hand-written HIP kernels behind a C-ABI shared library
(include/toploc.h); `binding` is the thin ctypes layer with the same names.
Importing this package does not load the library; the first call does, and
raises if it has not been built.
"""
