"""rv_block_update vs the definition w - eta*g in fp64 (paper Eq. 2), bar 1e-6."""
import numpy as np
import pytest
import torch

from paper_2401_01728_amd.inputs import gen
from util import dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [1, 5, 2047, 2048, 2049, 16576, 1000003])
@pytest.mark.parametrize("with_bf16", [False, True])
def test_update(n, with_bf16):
    import paper_2401_01728_amd as rv
    w = gen.normal_f32(11, 0, n, std=0.02)
    g = gen.normal_f32(11, 1, n, std=1e-3)
    eta = 1e-3 * 3
    dw, dg = dev(w), dev(g)
    copy = torch.zeros(n, dtype=torch.bfloat16, device="cuda") if with_bf16 else None
    rv.block_update(dw, dg, eta, bf16_out=copy)
    got = dw.cpu().numpy()
    ref = w.astype(np.float64) - np.float64(np.float32(eta)) * g.astype(np.float64)
    assert np.all(np.abs(got - ref) <= 1e-6 * (np.abs(w) + eta * np.abs(g)))
    assert np.array_equal(dg.cpu().numpy(), g)
    if with_bf16:
        bits = copy.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(bits, gen.f32_to_bf16_bits(got))      # rounding of the NEW weights


def test_update_unaligned():
    import paper_2401_01728_amd as rv
    n = 5001
    w = gen.normal_f32(12, 0, n); g = gen.normal_f32(12, 1, n)
    bw = torch.zeros(n + 4, device="cuda"); bg = torch.zeros(n + 4, device="cuda")
    vw, vg = bw[1:1 + n], bg[3:3 + n]
    vw.copy_(dev(w)); vg.copy_(dev(g))
    rv.block_update(vw, vg, 0.25)
    ref = w.astype(np.float64) - 0.25 * g.astype(np.float64)
    assert np.all(np.abs(vw.cpu().numpy() - ref) <= 1e-6 * (np.abs(w) + 0.25 * np.abs(g)))
    assert bw[0].item() == 0 and bw[n + 1].item() == 0
