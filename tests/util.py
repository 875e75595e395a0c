"""Helpers shared by the GPU parity tests (harness only: no method arithmetic)."""
import numpy as np
import torch

from paper_2401_01728_amd.inputs import gen


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def bf16_tensor_from_bits(bits, shape):
    """uint16 bit patterns -> torch bf16 CUDA tensor of the given shape."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda()
    return t.view(torch.bfloat16).reshape(shape)


def bf16_normal(seed, stream, shape, mean=0.0, std=1.0):
    """(torch bf16 CUDA tensor, the same values widened to fp64)."""
    n = int(np.prod(shape))
    bits = gen.normal_bf16_bits(seed, stream, n, mean, std)
    return bf16_tensor_from_bits(bits, shape), gen.bf16_bits_to_f32(bits).astype(np.float64).reshape(shape)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel(); b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def max_rel(a, b):
    a = np.asarray(a, dtype=np.float64).ravel(); b = np.asarray(b, dtype=np.float64).ravel()
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-300))
