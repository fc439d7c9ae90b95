"""MI355X-native hybrid decode path over asymmetric virtual-memory pools.

`inputs` holds the seeded synthetic workloads; `binding` is the thin ctypes
layer over the C-ABI library built from `csrc/` (it is imported on demand so
that the input generators stay usable without the native library).
"""
