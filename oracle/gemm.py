"""CPU oracle for the stage-load GEMM: C = A B^T in fp64.  Test infrastructure only.

The load generator multiplies bf16 matrices with fp32 accumulation and rounds the result to bf16; its definition is
the plain matrix product, so the oracle is that product evaluated in fp64 on the same (bf16-valued) inputs.
"""
import numpy as np


def gemm_nt(a, b):
    """a: [M, K], b: [N, K] (any float dtype holding bf16-representable values) -> fp64 [M, N] = a @ b.T."""
    return np.asarray(a, dtype=np.float64) @ np.asarray(b, dtype=np.float64).T
