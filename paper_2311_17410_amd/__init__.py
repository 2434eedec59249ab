"""MI355X-native temporal neighbourhood sampling (GNNFlow, arXiv 2311.17410, Algorithm 1).

``binding``    ctypes binding of the C ABI (include/tns.h); loads libtns.so lazily
``workloads``  seeded synthetic streams and query batches (no sampling arithmetic)
``build``      compiles the HIP library in-tree
"""
