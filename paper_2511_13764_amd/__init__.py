"""MI355X-native GEMM / batch-reduce GEMM (C = beta*C + sum_i A_i x B_i).

The compute lives in hand-written HIP kernels for gfx950 behind a C-ABI shared
library (csrc/, declared in include/brgemm.h); `binding` marshals arguments to
it.  Importing the package does not load the library; the first call does and
fails loudly if it has not been built.
"""
__all__ = ["binding", "workloads"]
