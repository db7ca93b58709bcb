"""MI355X-native layer-wise full-graph GNN inference (hot path of the DGI paper, arXiv 2211.15082).

The product is libdgi.so (C ABI in include/dgi.h, HIP kernels in csrc/); `binding` is its ctypes
wrapper.  Importing `binding` fails loudly when the library has not been built.
"""
__all__ = ["binding", "build"]
