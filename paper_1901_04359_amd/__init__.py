"""gTop-k S-SGD data-parallel hot path on MI355X (gfx950).

`workloads` draws the seeded synthetic inputs; `binding` is the thin ctypes
layer over the C-ABI library built from `csrc/` (it raises if the library is
missing: there is no CPU fallback).  Nothing is imported eagerly here, so the
input generators stay usable on a machine without the library.
"""
