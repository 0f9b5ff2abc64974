"""MI355X-native fused GEMM: C = act(alpha * A @ B + bias), hand-written HIP for gfx950.

``paper_2604_01489_amd.binding`` is the ctypes binding of the C-ABI library
(``include/gemm_epilogue.h``); ``paper_2604_01489_amd.inputs`` draws the seeded
synthetic workloads.  Importing the package loads neither torch nor the library.
"""
__all__ = ["binding", "inputs"]
