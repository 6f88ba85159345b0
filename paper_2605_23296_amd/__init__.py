"""MI355X-native batched block-compaction layer (HIP kernels behind a C ABI).

`workloads` draws seeded synthetic inputs; `binding` is the ctypes layer over
libcompact.so.  Importing the package loads nothing native; `binding.lib()`
does, and fails loudly when the library has not been built.
"""
