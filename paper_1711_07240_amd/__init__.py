"""libcgbn: Cross-GPU Batch Normalization hot path for MI355X (gfx950).

The compute lives in the HIP library under `csrc/`; `cgbn` is the thin
ctypes binding with the same names as the C ABI.  Importing this package does
not load the library; the binding loads it on first use and raises if it has
not been built.
"""
