"""Thin binding of include/rv_kernels.h (per-kernel entry points; marshalling only)."""
import ctypes

import torch

from . import _lib
from .api import _check, _ptr, _stream_handle

EPI_BF16, EPI_BF16_BIAS, EPI_F32_BIAS_RESID, EPI_BF16_BIAS_GELU, EPI_BF16_DGELU, EPI_F32, EPI_F32_BIAS_RESID_BF16 = range(7)


def gemm_bf16(A, a_kmajor, B, b_kmajor, M, N, K, epilogue, out, out2=None, bias=None, resid=None, zin=None,
              tile=0, stream=None):
    lda = A.stride(0); ldb = B.stride(0)
    _check(_lib.lib().rv_k_gemm_bf16(_ptr(A), lda, int(a_kmajor), _ptr(B), ldb, int(b_kmajor), M, N, K, epilogue,
                                     _ptr(out), out.stride(0), _ptr(out2), _ptr(bias), _ptr(resid),
                                     resid.stride(0) if resid is not None else 0, _ptr(zin), tile,
                                     _stream_handle(stream)))
    return out
