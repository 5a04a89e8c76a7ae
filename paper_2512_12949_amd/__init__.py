"""MI355X-native fused FFN (GEMM -> activation [-> gate] -> GEMM in one kernel).

``inputs`` holds the seeded synthetic workloads; ``binding`` the ctypes front end of the
C-ABI library ``libffuse.so`` (built from ``csrc/`` by ``build.py``).  The binding is
imported lazily so that the input generator can be used without the HIP library.
"""
