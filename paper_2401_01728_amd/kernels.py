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


def gemm_wgrad_grouped(xs, dys, outs, stream=None):
    """rv_k_gemm_wgrad_grouped: outs[i] (fp32 [M_i, N_i]) = xs[i]^T @ dys[i]; xs[i] is [K, M_i], dys[i] is [K, N_i]."""
    n = len(xs)
    K = xs[0].shape[0]
    vp = (ctypes.c_void_p * n); i64 = (ctypes.c_int64 * n); i32 = (ctypes.c_int * n)
    X = vp(*[_ptr(x) for x in xs]); Y = vp(*[_ptr(y) for y in dys]); O = vp(*[_ptr(o) for o in outs])
    lda = i64(*[x.stride(0) for x in xs]); ldb = i64(*[y.stride(0) for y in dys])
    M = i32(*[x.shape[1] for x in xs]); N = i32(*[y.shape[1] for y in dys])
    _check(_lib.lib().rv_k_gemm_wgrad_grouped(n, X, lda, Y, ldb, M, N, K, O, _stream_handle(stream)))
    return outs


def layernorm_fwd(x, gamma, beta, eps, xcopy=None, stream=None):
    T, d = x.shape
    y = torch.empty(T, d, dtype=torch.bfloat16, device="cuda")
    mean = torch.empty(T, dtype=torch.float32, device="cuda"); rstd = torch.empty_like(mean)
    _check(_lib.lib().rv_k_layernorm_fwd(_ptr(x), 1 if x.dtype == torch.bfloat16 else 0, _ptr(xcopy), _ptr(gamma),
                                         _ptr(beta), _ptr(y), _ptr(mean), _ptr(rstd), T, d, eps,
                                         _stream_handle(stream)))
    return y, mean, rstd


def layernorm_bwd(dy, x, mean, rstd, gamma, dres, want_bf16=True, stream=None):
    T, d = x.shape
    dx = torch.empty(T, d, dtype=torch.float32, device="cuda")
    dx16 = torch.empty(T, d, dtype=torch.bfloat16, device="cuda") if want_bf16 else None
    part = torch.empty(((T + 7) // 8) * 3 * d, dtype=torch.float32, device="cuda")
    dg, db, dbias = (torch.empty(d, dtype=torch.float32, device="cuda") for _ in range(3))
    _check(_lib.lib().rv_k_layernorm_bwd(_ptr(dy), _ptr(x), _ptr(mean), _ptr(rstd), _ptr(gamma), _ptr(dres),
                                         _ptr(dx), _ptr(dx16), _ptr(part), _ptr(dg), _ptr(db), _ptr(dbias), T, d,
                                         _stream_handle(stream)))
    return dx, dx16, dg, db, dbias


def attention_fwd(qkv, mb, S, d, H, stream=None):
    out = torch.empty(mb * S, d, dtype=torch.bfloat16, device="cuda")
    lse2 = torch.empty(mb * H * S, dtype=torch.float32, device="cuda")
    _check(_lib.lib().rv_k_attention_fwd(_ptr(qkv), _ptr(out), _ptr(lse2), mb, S, d, H, _stream_handle(stream)))
    return out, lse2


def attention_bwd(qkv, out, dout, lse2, mb, S, d, H, stream=None):
    dqkv = torch.full((mb * S, 3 * d), float("nan"), dtype=torch.bfloat16, device="cuda")
    scratch = torch.empty(mb * H * S, dtype=torch.float32, device="cuda")
    _check(_lib.lib().rv_k_attention_bwd(_ptr(qkv), _ptr(out), _ptr(dout), _ptr(lse2), _ptr(scratch), _ptr(dqkv),
                                         mb, S, d, H, _stream_handle(stream)))
    return dqkv


def attention_bwd_static(qkv, out, dout, lse2, dqkv, mb, S, d, H, stream=None):
    """rv_k_attention_bwd_static: dqkv is the caller's output; nothing is allocated here or in the library."""
    _check(_lib.lib().rv_k_attention_bwd_static(_ptr(qkv), _ptr(out), _ptr(dout), _ptr(lse2), _ptr(dqkv), mb, S, d,
                                                H, _stream_handle(stream)))
    return dqkv
