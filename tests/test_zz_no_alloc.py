"""The attention backward that allocates nothing (fixed scratch inside the library) against the
entry point that takes a caller workspace: same kernels, so the results must be identical bit
for bit; two calls in a row on one stream, the second on a smaller input, then the size limit."""
import numpy as np
import pytest
import torch

from util import bf16_normal

pytestmark = pytest.mark.gpu


def _case(seed, mb, S, H, dh):
    from paper_2401_01728_amd import kernels as k
    d = H * dh
    qkv, _ = bf16_normal(seed, 0, (mb * S, 3 * d), std=1.0)
    dout, _ = bf16_normal(seed, 1, (mb * S, d), std=1e-2)
    out, lse2 = k.attention_fwd(qkv, mb, S, d, H)
    ref = k.attention_bwd(qkv, out, dout, lse2, mb, S, d, H)
    got = torch.full((mb * S, 3 * d), float("nan"), dtype=torch.bfloat16, device="cuda")
    return (qkv, out, dout, lse2, got, mb, S, d, H), ref


def test_static_scratch_attention_backward_matches_workspace_variant():
    from paper_2401_01728_amd import kernels as k
    import paper_2401_01728_amd as rv
    big, ref_big = _case(11, 2, 512, 4, 64)       # 4096 scratch rows
    small, ref_small = _case(12, 1, 192, 2, 128)  # 384 rows: reuses the front of the same array
    k.attention_bwd_static(*big)
    k.attention_bwd_static(*small)
    torch.cuda.synchronize()
    for (args, ref) in ((big, ref_big), (small, ref_small)):
        got = args[4]
        assert not torch.isnan(got.float()).any()
        assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
    # beyond the fixed array: rejected, output untouched
    S = 64 * 1024
    z = torch.zeros(1, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(rv.RvError):
        k.attention_bwd_static(z, z, z, z.float(), z, 5, S, 64, 1)    # 5 * 65536 rows > 262144
