"""MI355X-native token-filtered decoder-layer backward (HIP, gfx950).

`workloads` holds the seeded synthetic input generators; `binding` is the thin
ctypes layer over the C-ABI library built from `csrc/`.  Importing the package
does not load the library; `binding.lib()` does, and fails loudly when it has
not been built.
"""
