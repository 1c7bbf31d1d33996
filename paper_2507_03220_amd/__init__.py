"""MI355X-native segmented base+adapter linear layer (Symbiosis, arXiv 2507.03220).

The product is the C-ABI library `libsymb.so` (see include/symb.h); `binding` is a thin
ctypes layer with the same entry-point names that marshals torch tensors into it.
Importing this package loads nothing; `binding.lib()` loads the library and fails
loudly if it has not been built.
"""
__all__ = ["binding", "build"]
