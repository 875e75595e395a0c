"""Device generator == host generator, bit for bit."""
import numpy as np
import pytest
import torch

from paper_2401_01728_amd.inputs import gen

pytestmark = pytest.mark.gpu


def test_device_fill_matches_host_bits():
    from paper_2401_01728_amd.inputs import device
    n = 100003
    t = torch.empty(n, dtype=torch.float32, device="cuda")
    device.fill_normal_(t, 9, 2, mean=0.5, std=0.02, offset=2**33)
    ref = gen.normal_f32(9, 2, n, mean=0.5, std=0.02, offset=2**33)
    assert np.array_equal(t.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    b = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    device.fill_normal_(b, 9, 3, std=1e-3)
    assert np.array_equal(b.view(torch.int16).cpu().numpy().view(np.uint16), gen.normal_bf16_bits(9, 3, n, std=1e-3))
    u = torch.empty(n, dtype=torch.float32, device="cuda")
    device.fill_uniform_(u, 9, 4, lo=-0.125, hi=0.125, offset=7)
    assert np.array_equal(u.cpu().numpy(), gen.uniform_f32(9, 4, n, -0.125, 0.125, offset=7))
