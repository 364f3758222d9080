"""MI355X-native 4-bit GELU activation path of S2A (Sec. 3.2, GeLU paragraph).

``s2a``        ctypes binding of the HIP library (the product path)
``workloads``  seeded synthetic inputs shared by tests and the benchmark
``build``      in-tree hipcc build of libs2a.so
"""
