"""MI355X-native decode attention for Multi-Head Low-Rank Attention (MLRA).

The compute path is the HIP library `libmlra.so` (C ABI declared in include/mlra.h), reached
through `paper_2603_02188_amd.binding`.  Importing this package does not load the library;
the binding loads it on first use and raises if it has not been built.
"""
__all__ = ["inputs", "roofline", "binding", "build"]
