"""flexgemm for MI355X: flexible mixed-precision GEMM and GETT contractions (arXiv 2009.12263).

``binding`` holds the ctypes front end of the C ABI (include/flexgemm.h); ``workloads`` the seeded
synthetic inputs; ``build`` compiles the HIP sources.  Nothing here computes on the CPU.
"""
