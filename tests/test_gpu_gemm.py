"""bf16 MFMA matrix products vs numpy fp64 on the same bf16-rounded operands.

Bar: bf16 outputs carry one bf16 rounding (2^-9 relative) on top of fp32 accumulation:
4e-3 (well inside the 2e-2 stage bar); fp32 outputs 1e-5; each normwise and element by element
(util.close).
"""
import numpy as np
import pytest
import torch

from oracle import blocks
from util import bf16_normal, close, host64, dev

pytestmark = pytest.mark.gpu

GROUP = {4e-3: "matrix product kernels, bf16 outputs", 1e-5: "matrix product kernels, fp32 outputs"}


def _out(shape, dtype):
    return torch.full(shape, float("nan"), dtype=dtype, device="cuda")


SHAPES = [(256, 256, 64), (128, 128, 128), (512, 384, 192), (200, 320, 256), (1024, 1024, 512), (64, 64, 64),
          (776, 1600, 320)]


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("tile", [2128, 2192, 2256, 5256])
def test_forward_product_and_epilogues(M, N, K, tile):
    from paper_2401_01728_amd import kernels as k
    x, x64 = bf16_normal(1, 0, (M, K))
    w, w64 = bf16_normal(1, 1, (K, N), std=0.05)
    b, b64 = bf16_normal(1, 2, (N,), std=0.5)
    r64 = np.random.default_rng(0).normal(size=(M, N)).astype(np.float32)
    r = dev(r64)
    ref = x64 @ w64 + b64
    o = _out((M, N), torch.bfloat16)
    k.gemm_bf16(x, 0, w, 1, M, N, K, k.EPI_BF16_BIAS, o, bias=b, tile=tile)
    close(host64(o), ref, 4e-3, "gemm", group=GROUP[4e-3])
    o32 = _out((M, N), torch.float32); o16 = _out((M, N), torch.bfloat16)
    k.gemm_bf16(x, 0, w, 1, M, N, K, k.EPI_F32_BIAS_RESID_BF16, o32, out2=o16, bias=b, resid=r, tile=tile)
    close(host64(o32), ref + r64, 1e-5, "gemm", group=GROUP[1e-5])
    close(host64(o16), ref + r64, 4e-3, "gemm", group=GROUP[4e-3])
    o32b = _out((M, N), torch.float32)
    k.gemm_bf16(x, 0, w, 1, M, N, K, k.EPI_F32_BIAS_RESID, o32b, bias=b, resid=r, tile=tile)
    assert torch.equal(o32, o32b)
    z = _out((M, N), torch.bfloat16); g = _out((M, N), torch.bfloat16)
    k.gemm_bf16(x, 0, w, 1, M, N, K, k.EPI_BF16_BIAS_GELU, z, out2=g, bias=b, tile=tile)
    close(host64(z), ref, 4e-3, "gemm", group=GROUP[4e-3])
    close(host64(g), blocks.gelu(ref), 4e-3, "gemm", group=GROUP[4e-3])


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("tile", [2128, 2192, 2256, 5256])
def test_input_gradient_product(M, N, K, tile):
    """dx[M, N] = dy[M, K] W^T with W stored [N, K] (its rows are the output columns)."""
    from paper_2401_01728_amd import kernels as k
    dy, dy64 = bf16_normal(2, 0, (M, K))
    w, w64 = bf16_normal(2, 1, (N, K), std=0.05)
    z, z64 = bf16_normal(2, 2, (M, N))
    ref = dy64 @ w64.T
    o = _out((M, N), torch.bfloat16)
    k.gemm_bf16(dy, 0, w, 0, M, N, K, k.EPI_BF16, o, tile=tile)
    close(host64(o), ref, 4e-3, "gemm", group=GROUP[4e-3])
    o2 = _out((M, N), torch.bfloat16)
    k.gemm_bf16(dy, 0, w, 0, M, N, K, k.EPI_BF16_DGELU, o2, zin=z, tile=tile)
    close(host64(o2), ref * blocks.gelu_grad(z64), 4e-3, "gemm", group=GROUP[4e-3])


@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("tile", [2128, 2192, 2256, 5256])
def test_weight_gradient_product(M, N, K, tile):
    """dW[M, N] = x^T dy with x [K, M] and dy [K, N]: contraction over the slow dimension."""
    from paper_2401_01728_amd import kernels as k
    x, x64 = bf16_normal(3, 0, (K, M))
    dy, dy64 = bf16_normal(3, 1, (K, N))
    o = _out((M, N), torch.float32)
    k.gemm_bf16(x, 1, dy, 1, M, N, K, k.EPI_F32, o, tile=tile)
    close(host64(o), x64.T @ dy64, 1e-5, "gemm", group=GROUP[1e-5])


@pytest.mark.parametrize("K", [64, 128, 192, 256, 320, 384, 448, 576])
def test_ring_depths_of_the_256_tile(K):
    """The 256x256 tile walks K through a four-slot ring of 32-deep tiles (K/32 = 2 .. 18 tiles:
    fewer tiles than slots, exactly as many, one more, and a few turns of the ring), each layout,
    on a ragged output (two tile rows, two tile columns, the last of each partly filled)."""
    from paper_2401_01728_amd import kernels as k
    M, N = 328, 456
    x, x64 = bf16_normal(11, 0, (M, K)); w, w64 = bf16_normal(11, 1, (K, N), std=0.05)
    b, b64 = bf16_normal(11, 2, (N,), std=0.5)
    o = _out((M, N), torch.bfloat16)
    k.gemm_bf16(x, 0, w, 1, M, N, K, k.EPI_BF16_BIAS, o, bias=b, tile=5256)            # forward layout
    close(host64(o), x64 @ w64 + b64, 4e-3, "gemm", group=GROUP[4e-3])
    wt, wt64 = bf16_normal(11, 3, (N, K), std=0.05)
    o = _out((M, N), torch.bfloat16)
    k.gemm_bf16(x, 0, wt, 0, M, N, K, k.EPI_BF16, o, tile=5256)                         # input-gradient layout
    close(host64(o), x64 @ wt64.T, 4e-3, "gemm", group=GROUP[4e-3])
    xt, xt64 = bf16_normal(11, 4, (K, M)); dy, dy64 = bf16_normal(11, 5, (K, N), std=1e-2)
    o32 = _out((M, N), torch.float32)
    k.gemm_bf16(xt, 1, dy, 1, M, N, K, k.EPI_F32, o32, tile=5256)                       # weight-gradient layout
    close(host64(o32), xt64.T @ dy64, 1e-5, "gemm", group=GROUP[1e-5])
    g32 = _out((M, N), torch.float32)
    k.gemm_wgrad_grouped([xt], [dy], [g32])
    assert torch.equal(g32, o32)


def test_strided_operands_and_rejects():
    """Operands that are column blocks of wider matrices (pitch > width), as q|k|v are."""
    from paper_2401_01728_amd import kernels as k
    import paper_2401_01728_amd as rv
    M, N, K = 256, 192, 128
    big, big64 = bf16_normal(4, 0, (M, 3 * K))
    w, w64 = bf16_normal(4, 1, (K, N), std=0.05)
    b, b64 = bf16_normal(4, 2, (N,))
    x = big[:, K:2 * K]
    o = _out((M, N), torch.bfloat16)
    k.gemm_bf16(x, 0, w, 1, M, N, K, k.EPI_BF16_BIAS, o, bias=b)
    close(host64(o), big64[:, K:2 * K] @ w64 + b64, 4e-3, "gemm", group=GROUP[4e-3])
    with pytest.raises(rv.RvError):
        k.gemm_bf16(x, 0, w, 1, M, N, 100, k.EPI_BF16_BIAS, o, bias=b)       # K % 64
    with pytest.raises(rv.RvError):
        k.gemm_bf16(x, 1, w, 0, M, N, K, k.EPI_BF16, o)                      # unsupported layout pair
    wide = _out((M, N + 4), torch.bfloat16)
    with pytest.raises(rv.RvError):
        k.gemm_bf16(x, 0, w, 1, M, N, K, k.EPI_BF16_BIAS, wide[:, :N], bias=b)   # bf16 output pitch % 8


def test_grouped_weight_gradient_products():
    """Four products of different widths in one launch equal the single launches bit for bit."""
    from paper_2401_01728_amd import kernels as k
    K = 320
    dims = [(192, 256), (64, 64), (136, 512), (512, 72)]
    xs, dys, outs, refs = [], [], [], []
    for i, (M, N) in enumerate(dims):
        x, x64 = bf16_normal(9, 2 * i, (K, M)); dy, dy64 = bf16_normal(9, 2 * i + 1, (K, N), std=1e-2)
        xs.append(x); dys.append(dy); outs.append(_out((M, N), torch.float32)); refs.append(x64.T @ dy64)
    k.gemm_wgrad_grouped(xs, dys, outs)
    for i, (M, N) in enumerate(dims):
        close(host64(outs[i]), refs[i], 1e-5, "gemm", group=GROUP[1e-5])
        single = _out((M, N), torch.float32)
        k.gemm_bf16(xs[i], 1, dys[i], 1, M, N, K, k.EPI_F32, single, tile=5256)
        assert torch.equal(single, outs[i])
    import paper_2401_01728_amd as rv
    with pytest.raises(rv.RvError):
        k.gemm_wgrad_grouped(xs * 2, dys * 2, outs * 2)      # more than four
