"""MI355X-native LLVQ inference hot path: thin Python binding over the C ABI of libllvq.so.

Every step of the path (index decode, shape-gain scaling, fused matrix product) runs in the HIP kernels
of csrc/; this package only marshals torch device tensors into the C calls declared in include/llvq.h.
"""
from .binding import (LLVQ, LLVQError, lib_path, build_library, LLVQ_IDX_U48, LLVQ_IDX_U64, LLVQ_IDX_U24,
                      LLVQ_F16, LLVQ_BF16, LLVQ_F32, LLVQ_ANGULAR, LLVQ_EUCLIDEAN)

__all__ = ["LLVQ", "LLVQError", "lib_path", "build_library", "LLVQ_IDX_U48", "LLVQ_IDX_U64", "LLVQ_IDX_U24",
           "LLVQ_F16", "LLVQ_BF16", "LLVQ_F32", "LLVQ_ANGULAR", "LLVQ_EUCLIDEAN"]
