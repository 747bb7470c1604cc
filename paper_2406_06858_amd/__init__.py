"""MI355X-native fused tensor-parallel GEMMs (GEMM-ReduceScatter, AllGather-GEMM).

The compute path is the C-ABI library built from `csrc/`; `binding` marshals arguments to it.
Importing the package does not load the library; the first call does, and raises if the
library has not been built.
"""
__all__ = ["binding", "inputs"]
