"""Thin Python binding of include/rv.h: argument marshalling only.

torch is used for device memory and streams; every step of the path runs in librv.so.
"""
import ctypes

import torch

from . import _lib

RV_MLP, RV_DECODER = 0, 1
RV_F32, RV_BF16 = 0, 1
RV_OK, RV_E_INVAL, RV_E_STASH_FULL, RV_E_UNKNOWN_MB, RV_E_DUP_MB, RV_E_NOMEM, RV_E_DEVICE = (
    0, -1, -2, -3, -4, -5, -6)


class RvError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__("rv: %s (%d)" % (_lib.lib().rv_strerror(status).decode(), status))


def _check(status):
    if status != RV_OK:
        raise RvError(status)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_f32(t, n=None):
    assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
    if n is not None:
        assert t.numel() == n
    return t


class Stage:
    """rv_stage_* : one peer's block with tau+1 stash slots and weight versions."""

    def __init__(self, kind, dims, n_layers, microbatch, tau, eta, ln_eps=1e-5, stream=None):
        self._h = None
        self.kind = kind
        self.dims = [int(x) for x in dims]
        self.microbatch = int(microbatch)
        arr = (ctypes.c_int64 * len(self.dims))(*self.dims)
        d = _lib.StageDesc(kind, RV_F32 if kind == RV_MLP else RV_BF16, n_layers, arr, microbatch, tau,
                           eta, ln_eps, _stream_handle(stream))
        h = ctypes.c_void_p()
        _check(_lib.lib().rv_stage_create(ctypes.byref(d), ctypes.byref(h)))
        self._h = h
        self.act_dtype = torch.float32 if kind == RV_MLP else torch.bfloat16
        if kind == RV_MLP:
            self.in_shape, self.out_shape = (microbatch, self.dims[0]), (microbatch, self.dims[-1])
        else:
            self.in_shape = self.out_shape = (microbatch, self.dims[3], self.dims[0])

    @classmethod
    def mlp(cls, dims, microbatch, tau, eta, stream=None):
        return cls(RV_MLP, dims, len(dims) - 1, microbatch, tau, eta, stream=stream)

    @classmethod
    def decoder(cls, n_blocks, d_model, n_heads, d_ffn, seq, microbatch, tau, eta, ln_eps=1e-5, stream=None,
                keep_grad=False):
        st = cls(RV_DECODER, [d_model, n_heads, d_ffn, seq], n_blocks, microbatch, tau, eta, ln_eps, stream)
        if keep_grad:
            st.keep_grad(True)
        return st

    def close(self):
        if self._h is not None:
            _lib.lib().rv_stage_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def num_params(self):
        return int(_lib.lib().rv_stage_num_params(self._h))

    @property
    def in_flight(self):
        return int(_lib.lib().rv_stage_in_flight(self._h))

    def set_params(self, flat):
        _check(_lib.lib().rv_stage_set_params(self._h, _ptr(_dev_f32(flat)), flat.numel()))

    def set_optimizer(self, momentum=0.0, weight_decay=0.0):
        _check(_lib.lib().rv_stage_set_optimizer(self._h, momentum, weight_decay))

    def set_accumulation(self, microbatches):
        _check(_lib.lib().rv_stage_set_accumulation(self._h, int(microbatches)))

    def keep_grad(self, on=True):
        _check(_lib.lib().rv_stage_keep_grad(self._h, 1 if on else 0))

    def defer_update(self, on=True):
        _check(_lib.lib().rv_stage_defer_update(self._h, 1 if on else 0))

    def get_params(self, out=None):
        if out is None:
            out = torch.empty(self.num_params, dtype=torch.float32, device="cuda")
        _check(_lib.lib().rv_stage_get_params(self._h, _ptr(_dev_f32(out)), out.numel()))
        return out

    def last_grad(self, out=None):
        if out is None:
            out = torch.empty(self.num_params, dtype=torch.float32, device="cuda")
        _check(_lib.lib().rv_stage_last_grad(self._h, _ptr(_dev_f32(out)), out.numel()))
        return out

    def profile(self, on=True):
        _check(_lib.lib().rv_stage_profile(self._h, 1 if on else 0))

    def profile_read(self):
        """(launches, mean microseconds) of the grouped weight-gradient launches bracketed so far."""
        n, us = ctypes.c_int(0), ctypes.c_float(0.0)
        _check(_lib.lib().rv_stage_profile_read(self._h, ctypes.byref(n), ctypes.byref(us)))
        return n.value, us.value

    def _act(self, t, shape):
        assert t.is_cuda and t.dtype == self.act_dtype and t.is_contiguous() and tuple(t.shape) == tuple(shape), \
            (t.dtype, tuple(t.shape), shape)
        return t

    def forward(self, mb_id, x, out=None):
        if out is None:
            out = torch.empty(self.out_shape, dtype=self.act_dtype, device="cuda")
        _check(_lib.lib().rv_stage_forward(self._h, mb_id, _ptr(self._act(x, self.in_shape)),
                                           _ptr(self._act(out, self.out_shape))))
        return out

    def backward(self, mb_id, grad_out, grad_in=None, want_grad_in=True):
        if grad_in is None and want_grad_in:
            grad_in = torch.empty(self.in_shape, dtype=self.act_dtype, device="cuda")
        if grad_in is not None:
            self._act(grad_in, self.in_shape)
        _check(_lib.lib().rv_stage_backward(self._h, mb_id, _ptr(self._act(grad_out, self.out_shape)),
                                            _ptr(grad_in)))
        return grad_in


def _stage_step(self, fwd_mb, x, bwd_mb, grad_out, out=None, grad_in=None):
    """rv_stage_step: forward(fwd_mb) beside backward(bwd_mb), then the update."""
    if out is None:
        out = torch.empty(self.out_shape, dtype=self.act_dtype, device="cuda")
    if grad_in is None:
        grad_in = torch.empty(self.in_shape, dtype=self.act_dtype, device="cuda")
    _check(_lib.lib().rv_stage_step(self._h, fwd_mb, _ptr(self._act(x, self.in_shape)),
                                    _ptr(self._act(out, self.out_shape)), bwd_mb,
                                    _ptr(self._act(grad_out, self.out_shape)),
                                    _ptr(self._act(grad_in, self.in_shape))))
    return out, grad_in


Stage.step = _stage_step


def block_update(w, g, eta, bf16_out=None, stream=None):
    """rv_block_update: w <- w - eta*g in place (fp32), optional bf16 copy."""
    _dev_f32(w); _dev_f32(g, w.numel())
    if bf16_out is not None:
        assert bf16_out.is_cuda and bf16_out.dtype == torch.bfloat16 and bf16_out.numel() == w.numel()
    _check(_lib.lib().rv_block_update(_ptr(w), _ptr(g), w.numel(), eta, _ptr(bf16_out), _stream_handle(stream)))


def block_update_momentum(w, g, v, eta, momentum, weight_decay, bf16_out=None, stream=None):
    """rv_block_update_momentum: in-place momentum / weight-decay step on fp32 vectors."""
    _dev_f32(w); _dev_f32(g, w.numel()); _dev_f32(v, w.numel())
    _check(_lib.lib().rv_block_update_momentum(_ptr(w), _ptr(g), _ptr(v), w.numel(), eta, momentum, weight_decay,
                                               _ptr(bf16_out), _stream_handle(stream)))


def cluster_sync(stages, R, pending=-1):
    """rv_cluster_sync: every stage's parameters become their ring-partitioned mean (Alg. 2)."""
    import ctypes
    arr = (ctypes.c_void_p * len(stages))(*[s._h for s in stages])
    _check(_lib.lib().rv_cluster_sync(arr, len(stages), R, pending))


def cluster_sync_fork(stages, R, pending=-1, average_state=False, stream=None):
    """rv_cluster_sync_fork: the averaging on `stream` (a torch stream) beside the stages' own."""
    arr = (ctypes.c_void_p * len(stages))(*[s._h for s in stages])
    _check(_lib.lib().rv_cluster_sync_fork(arr, len(stages), R, pending, 1 if average_state else 0,
                                           _stream_handle(stream)))


def cluster_sync_join(stages):
    arr = (ctypes.c_void_p * len(stages))(*[s._h for s in stages])
    _check(_lib.lib().rv_cluster_sync_join(arr, len(stages)))


def cluster_average(replicas, R, mean_out=None, write_back=False, grad=None, grad_replica=0, eta=0.0,
                    stream=None, ring_offsets=None):
    """rv_cluster_average over a list of fp32 device vectors (rv_cluster_average_v when
    ring_offsets, R+1 element offsets, is given)."""
    C = len(replicas)
    n = replicas[0].numel() if C else 0
    for r in replicas:
        _dev_f32(r, n)
    if mean_out is not None:
        _dev_f32(mean_out, n)
    if grad is not None:
        _dev_f32(grad, n)
    arr = (ctypes.c_void_p * max(C, 1))(*[r.data_ptr() for r in replicas])
    if ring_offsets is not None:
        offs = (ctypes.c_int64 * len(ring_offsets))(*[int(o) for o in ring_offsets])
        _check(_lib.lib().rv_cluster_average_v(arr, C, n, offs, len(ring_offsets) - 1, _ptr(mean_out),
                                               1 if write_back else 0, _ptr(grad), grad_replica, eta,
                                               _stream_handle(stream)))
        return mean_out
    _check(_lib.lib().rv_cluster_average(arr, C, n, R, _ptr(mean_out), 1 if write_back else 0, _ptr(grad),
                                         grad_replica, eta, _stream_handle(stream)))
    return mean_out
