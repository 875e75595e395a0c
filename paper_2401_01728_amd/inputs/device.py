"""Device-side fills of the seeded generator (bit-identical to gen.py)."""
import ctypes

import torch

from .. import _lib
from . import gen


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def fill_normal_(t, seed, stream, mean=0.0, std=1.0, offset=0):
    """In-place fill of an fp32 or bf16 contiguous CUDA tensor (flat element order)."""
    assert t.is_cuda and t.is_contiguous() and t.dtype in (torch.float32, torch.bfloat16)
    rc = _lib.genlib().rvgen_fill_normal(ctypes.c_void_p(t.data_ptr()), t.numel(), seed, stream, mean, std,
                                         offset, float(gen.NORMAL_SCALE), 1 if t.dtype == torch.bfloat16 else 0,
                                         _stream())
    if rc != 0:
        raise RuntimeError("rvgen_fill_normal failed (%d)" % rc)
    return t


def fill_uniform_(t, seed, stream, lo=0.0, hi=1.0, offset=0):
    assert t.is_cuda and t.is_contiguous() and t.dtype == torch.float32
    rc = _lib.genlib().rvgen_fill_uniform(ctypes.c_void_p(t.data_ptr()), t.numel(), seed, stream, lo, hi, offset,
                                          _stream())
    if rc != 0:
        raise RuntimeError("rvgen_fill_uniform failed (%d)" % rc)
    return t
