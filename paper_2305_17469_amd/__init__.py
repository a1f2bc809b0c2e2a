"""MI355X-native GNN aggregation / combination hot path (GraphTensor, arXiv 2305.17469).

The product is libgt.so (C ABI in include/gt.h, HIP kernels in csrc/); `binding` exposes the same
entry points to Python.  `python -m paper_2305_17469_amd.build` compiles the library.
"""
__all__ = ["binding", "build", "feed", "stack"]
