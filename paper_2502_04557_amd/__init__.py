"""MI355X-native batched SPRINTER decode step (hand-written HIP behind a C ABI).

The package holds the HIP/C++ sources (csrc/), the in-tree build helper and a
thin ctypes binding whose functions mirror include/sprinter.h one to one.
Importing the package does not load the shared library; `binding.load_library()`
does, and raises if it has not been built.
"""
