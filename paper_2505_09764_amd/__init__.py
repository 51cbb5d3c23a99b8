"""MI355X-native batched All-to-All(v) schedule synthesis (FAST, arxiv 2505.09764).

binding    ctypes binding of libfast.so, the C ABI declared in include/fast.h
workloads  seeded synthetic traffic matrices (input data only)
build      compiles the native libraries in-tree with hipcc for gfx950
"""
