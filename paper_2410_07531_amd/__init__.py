"""MI355X-native RNG/GEMM overlap for attention dropout (arxiv 2410.07531 hot path).

The product is the C-ABI shared library built from `csrc/`; `binding` is a thin
ctypes layer over it.  Nothing is loaded at import time.
"""
