"""MI355X-native horizontally fused training-array operators (HFTA hot path).

``paper_2102_02344_amd.binding`` is the ctypes binding over the C ABI declared in
``include/hfta.h``; ``paper_2102_02344_amd.build`` compiles the HIP sources into
``libhfta.so`` in-tree.  Importing this package does not load the library.
"""
__all__ = ["binding", "build", "arrays"]
