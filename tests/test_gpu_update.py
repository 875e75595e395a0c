"""rv_block_update vs the oracle's update (oracle/stage.py: Eq. 2 and its momentum variant) in fp64, bar 1e-6."""
import numpy as np
import pytest
import torch

from oracle import stage as ostage
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
    ref = ostage.sgd_step(w.astype(np.float64), g.astype(np.float64), np.float64(np.float32(eta)))
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
    ref = ostage.sgd_step(w.astype(np.float64), g.astype(np.float64), 0.25)
    assert np.all(np.abs(vw.cpu().numpy() - ref) <= 1e-6 * (np.abs(w) + 0.25 * np.abs(g)))
    assert bw[0].item() == 0 and bw[n + 1].item() == 0


@pytest.mark.parametrize("n", [5, 2049, 1000003])
def test_momentum_update(n):
    """d = g + wd w; v <- mu v + d; w <- w - eta v (section 4.1 optimiser) vs fp64, 1e-6 bar."""
    import paper_2401_01728_amd as rv
    w = gen.normal_f32(13, 0, n, std=0.02); g = gen.normal_f32(13, 1, n, std=1e-3); v = gen.normal_f32(13, 2, n, std=1e-3)
    eta, mu, wd = 0.01, 0.9, 5e-4
    dw, dg, dv = dev(w), dev(g), dev(v)
    copy = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    rv.block_update_momentum(dw, dg, dv, eta, mu, wd, bf16_out=copy)
    f = lambda a: np.float64(np.float32(a))
    w_ref, v_ref = ostage.momentum_step(w.astype(np.float64), g.astype(np.float64), v.astype(np.float64), f(eta), f(mu), f(wd))
    gv, gw = dv.cpu().numpy(), dw.cpu().numpy()
    assert np.all(np.abs(gv - v_ref) <= 1e-6 * (np.abs(v) + np.abs(g) + wd * np.abs(w)))
    assert np.all(np.abs(gw - w_ref) <= 1e-6 * (np.abs(w) + eta * np.abs(v_ref)))
    assert np.array_equal(copy.view(torch.int16).cpu().numpy().view(np.uint16), gen.f32_to_bf16_bits(gw))
    # mu = wd = 0 is the plain step, bit for bit
    a, b = dev(w), dev(w); z = torch.zeros(n, device="cuda")
    rv.block_update_momentum(a, dg, z, eta, 0.0, 0.0); rv.block_update(b, dg, eta)
    assert torch.equal(a, b)
