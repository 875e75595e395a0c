"""LayerNorm and causal attention kernels vs the oracle's definitions
(fp64 on the same bf16-rounded inputs).  Bars: bf16 outputs 4e-3 (one bf16 rounding on fp32
arithmetic; attention 8e-3 / 1e-2: probabilities are rounded to bf16 before the second
product), fp32 outputs 1e-5; each normwise and element by element (util.close)."""
import numpy as np
import pytest
import torch

from oracle import blocks
from paper_2401_01728_amd.inputs import gen
from util import bf16_normal, close, host64, dev

pytestmark = pytest.mark.gpu


# the last three rows: 8192 rows and more take the four-rows-per-wave forward (seven and four column
# groups), 1792 is the widest row of the two-register-set forward
@pytest.mark.parametrize("T,d", [(64, 128), (100, 1024), (37, 1600), (16, 2048), (8, 4096), (5, 64),
                                 (8203, 1600), (8197, 1024), (23, 1792)])
def test_layernorm_forward_backward(T, d):
    from paper_2401_01728_amd import kernels as k
    eps = 1e-5
    x32 = gen.normal_f32(1, 0, T * d, mean=0.3, std=2.0).reshape(T, d)
    g, g64 = bf16_normal(1, 1, (d,), mean=1.0, std=0.1)
    b, b64 = bf16_normal(1, 2, (d,), std=0.1)
    y, mean, rstd = k.layernorm_fwd(dev(x32), g, b, eps)
    ref, (xh, r) = blocks.layernorm_fwd(x32.astype(np.float64), g64, b64, eps)
    close(host64(y), ref, 4e-3, "k", group="LayerNorm / column sum / attention kernels, bar 4e-3")
    close(host64(mean), x32.astype(np.float64).mean(-1), 1e-5, "k", group="LayerNorm / column sum / attention kernels, bar 1e-5")
    close(host64(rstd), r[:, 0], 1e-5, "k", group="LayerNorm / column sum / attention kernels, bar 1e-5")
    # bf16 input variant also emits the widened copy
    xb, xb64 = bf16_normal(1, 3, (T, d), std=1.5)
    xc = torch.empty(T, d, dtype=torch.float32, device="cuda")
    y2, _, _ = k.layernorm_fwd(xb, g, b, eps, xcopy=xc)
    assert np.array_equal(host64(xc), xb64)
    close(host64(y2), blocks.layernorm_fwd(xb64, g64, b64, eps)[0], 4e-3, "k", group="LayerNorm / column sum / attention kernels, bar 4e-3")
    # backward joined with the residual branch
    dy, dy64 = bf16_normal(1, 4, (T, d), std=1e-2)
    dres32 = gen.normal_f32(1, 5, T * d, std=1e-2).reshape(T, d)
    dx, dx16, dg, db, dbias = k.layernorm_bwd(dy, dev(x32), mean, rstd, g, dev(dres32))
    rdx, rdg, rdb = blocks.layernorm_bwd(dy64, g64, (xh, r))
    rdx = rdx + dres32
    close(host64(dx), rdx, 1e-5, "k", group="LayerNorm / column sum / attention kernels, bar 1e-5")
    close(host64(dx16), rdx, 4e-3, "k", group="LayerNorm / column sum / attention kernels, bar 4e-3")
    close(host64(dg), rdg, 1e-5, "k", group="LayerNorm / column sum / attention kernels, bar 1e-5")
    close(host64(db), rdb, 1e-5, "k", group="LayerNorm / column sum / attention kernels, bar 1e-5")
    close(host64(dbias), rdx.sum(0), 1e-5, "k", group="LayerNorm / column sum / attention kernels, bar 1e-5")


def _heads(t64, mb, S, H, dh):
    return t64.reshape(mb, S, H, dh).transpose(0, 2, 1, 3)


def _unheads(t):
    mb, H, S, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(mb * S, H * dh)


@pytest.mark.parametrize("mb,S,H,dh", [(2, 128, 2, 64), (1, 192, 3, 64), (1, 256, 2, 128), (2, 512, 2, 64),
                                        (1, 64, 1, 64), (1, 320, 1, 128)])
def test_attention_forward_backward(mb, S, H, dh):
    from paper_2401_01728_amd import kernels as k
    d = H * dh
    qkv, qkv64 = bf16_normal(3, 0, (mb * S, 3 * d), std=1.0)
    q, kk, v = (_heads(qkv64[:, i * d:(i + 1) * d], mb, S, H, dh) for i in range(3))
    ref, prob = blocks.causal_attention_fwd(q, kk, v)
    out, lse2 = k.attention_fwd(qkv, mb, S, d, H)
    close(host64(out), _unheads(ref), 8e-3, "k", group="LayerNorm / column sum / attention kernels, bar 8e-3")
    # log-sum-exp (base 2, scaled domain) against the definition
    s = np.einsum("bhid,bhjd->bhij", q, kk) / np.sqrt(dh)
    s = np.where(np.tril(np.ones((S, S), bool)), s, -np.inf)
    mx = s.max(-1)
    lse_ref = (mx + np.log(np.exp(s - mx[..., None]).sum(-1))) / np.log(2.0)
    assert np.abs(host64(lse2).reshape(mb, H, S) - lse_ref).max() < 1e-3
    dout, dout64 = bf16_normal(3, 1, (mb * S, d), std=1e-2)
    dq, dk, dv = blocks.causal_attention_bwd(_heads(dout64, mb, S, H, dh), q, kk, v, prob)
    # the kernel's D = rowsum(dO * O) uses its own bf16 output, as the stage does
    dqkv = host64(k.attention_bwd(qkv, out, dout, lse2, mb, S, d, H))
    close(dqkv[:, :d], _unheads(dq), 1e-2, "k", group="LayerNorm / column sum / attention kernels, bar 1e-2")
    close(dqkv[:, d:2 * d], _unheads(dk), 1e-2, "k", group="LayerNorm / column sum / attention kernels, bar 1e-2")
    close(dqkv[:, 2 * d:], _unheads(dv), 8e-3, "k", group="LayerNorm / column sum / attention kernels, bar 8e-3")


def test_attention_rejects_unsupported_shapes():
    from paper_2401_01728_amd import kernels as k
    import paper_2401_01728_amd as rv
    qkv = torch.zeros(100, 3 * 96, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rv.RvError):
        k.attention_fwd(qkv, 1, 100, 96, 1)        # head size 96, seq 100
