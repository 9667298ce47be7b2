"""ABFT-checked u8 x s8 -> s32 GEMM for MI355X (gfx950).

Hot path of arXiv 2103.00130, Section IV / Algorithm 1: the weight matrix is
packed once together with its checksum column B e, and every product row is
verified against A (B e) inside the same int8-MFMA pass, before requantization.
All arithmetic runs in the HIP kernels behind the C ABI declared in
include/abft_gemm.h; `binding` only marshals arguments.
"""
from . import workloads  # noqa: F401

__all__ = ["workloads"]
