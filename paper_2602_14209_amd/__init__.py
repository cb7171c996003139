"""MI355X-native hot path of MAGE ([MASK]-Guided Sparse Attention, arxiv 2602.14209).

``binding``   ctypes front end of the C-ABI HIP library (libmage.so)
``workloads`` seeded synthetic inputs
``build``     in-tree hipcc build of the library
"""
__all__ = ["binding", "workloads", "build"]
