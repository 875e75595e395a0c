"""rv_cluster_average vs the oracle (paper section 3.2; Alg. 2 all-reduce branch; Eq. 17).

Two bars: (i) against the fp64 direct mean, component-wise |err| <= 1e-6 * mean_c|x_c[i]|
(+ eta|g|/C when a gradient is folded in) and 1e-6 normwise; (ii) bit-exact against the
oracle's fp32 ring-order twin, since both sides take the additions in the ring's order.
"""
import numpy as np
import pytest
import torch

from oracle import average
from paper_2401_01728_amd.inputs import gen
from util import dev, rel_l2

pytestmark = pytest.mark.gpu


def _replicas(seed, C, n, shared_std=1.0, noise_std=1.0):
    o = gen.normal_f32(seed, 0, n, std=shared_std)
    return [(o + gen.normal_f32(seed, 1 + c, n, std=noise_std)).astype(np.float32) for c in range(C)]


def _check(xs, R, grad, gr, eta, write_back):
    import paper_2401_01728_amd as rv
    C, n = len(xs), xs[0].size
    dx = [dev(x) for x in xs]
    out = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    dg = dev(grad) if grad is not None else None
    rv.cluster_average(dx, R, mean_out=out, write_back=write_back, grad=dg, grad_replica=gr, eta=eta)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    ref = average.direct_mean(xs, grad, gr, eta)
    bound = 1e-6 * np.mean(np.abs(np.stack(xs)).astype(np.float64), axis=0)
    if grad is not None:
        bound = bound + 1e-6 * abs(eta) * np.abs(grad.astype(np.float64)) / C
    assert np.all(np.abs(got.astype(np.float64) - ref) <= bound)
    assert rel_l2(got, ref) <= 1e-6
    twin = average.ring_order_mean_f32(xs, R, grad, gr, eta)
    assert np.array_equal(got.view(np.uint32), twin.view(np.uint32))
    for c in range(C):
        after = dx[c].cpu().numpy()
        assert np.array_equal(after, got if write_back else xs[c])


@pytest.mark.parametrize("C,R,n", [
    (2, 2, 16576),            # config 1: one MLP stage's vector
    (4, 4, 50000 + 3),        # several tiles, ragged tail
    (8, 4, 3 * 2048 + 1),
    (16, 8, 40000),
    (16, 1, 4099), (3, 2, 10001), (5, 3, 7777), (7, 5, 64), (1, 1, 1000), (2, 7, 5),
    (16, 8, 100), (64, 3, 3000),
])
@pytest.mark.parametrize("fused", [False, True])
def test_average_matches_oracle(C, R, n, fused):
    xs = _replicas(40 + C, C, n)
    g = gen.normal_f32(40 + C, 99, n, std=1e-3) if fused else None
    _check(xs, R, g, (C - 1) if fused else 0, 1e-3 * 37, write_back=False)


@pytest.mark.parametrize("C,R,n", [(4, 4, 50003), (16, 2, 9000), (3, 3, 100)])
def test_average_write_back(C, R, n):
    xs = _replicas(7, C, n)
    g = gen.normal_f32(7, 99, n, std=1e-3)
    _check(xs, R, g, 0, 0.5, write_back=True)
    _check(xs, R, None, 0, 0.0, write_back=True)


def test_average_unaligned_pointers():
    import paper_2401_01728_amd as rv
    C, n, R = 4, 20001, 3
    xs = _replicas(8, C, n)
    big = [torch.zeros(n + 8, dtype=torch.float32, device="cuda") for _ in range(C)]
    views = []
    for c in range(C):
        v = big[c][1 + c % 3:1 + c % 3 + n]
        v.copy_(dev(xs[c])); views.append(v)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    rv.cluster_average(views, R, mean_out=out)
    assert np.array_equal(out.cpu().numpy(), average.ring_order_mean_f32(xs, R))


def test_identical_replicas_and_eq17():
    import paper_2401_01728_amd as rv
    n, C = 30000, 8
    x = gen.normal_f32(3, 0, n)
    g = gen.normal_f32(3, 1, n)
    reps = [dev(x) for _ in range(C)]
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    rv.cluster_average(reps, 4, mean_out=out)
    got = out.cpu().numpy()
    # a left fold of equal terms rounds from 3x on: at most C-1 roundings of 2^-24
    assert np.all(np.abs(got.astype(np.float64) - x) <= (C - 1) * 2.0**-24 * np.abs(x))
    assert np.array_equal(got, average.ring_order_mean_f32([x] * C, 4))
    pair = torch.empty(n, dtype=torch.float32, device="cuda")
    rv.cluster_average(reps[:2], 2, mean_out=pair)
    assert np.array_equal(pair.cpu().numpy(), x)         # C = 2: x + x and /2 are exact
    out2 = torch.empty(n, dtype=torch.float32, device="cuda")
    rv.cluster_average(reps, 4, mean_out=out2, grad=dev(g), grad_replica=3, eta=0.5)
    d = out2.cpu().numpy().astype(np.float64) - x
    assert np.allclose(d, -(0.5 / C) * g.astype(np.float64), rtol=0, atol=2e-6)


def test_average_rejects_bad_arguments():
    import paper_2401_01728_amd as rv
    a = torch.zeros(16, device="cuda"); b = torch.zeros(16, device="cuda")
    with pytest.raises(rv.RvError):
        rv.cluster_average([a, b], 0, mean_out=torch.zeros(16, device="cuda"))
    with pytest.raises(rv.RvError):
        rv.cluster_average([a, a], 1, mean_out=torch.zeros(16, device="cuda"))
    with pytest.raises(rv.RvError):
        rv.cluster_average([a, b], 1, mean_out=a)
    with pytest.raises(rv.RvError):
        rv.cluster_average([a, b], 1, mean_out=None, write_back=False)


@pytest.mark.parametrize("C,offs", [
    (4, [0, 10001, 10001, 30007, 50003]),           # unequal, unaligned boundaries, an empty ring
    (16, [0, 4096, 12288, 40000]),
    (3, [0, 1, 2, 3, 9999]),
    (8, [0, 100000]),
])
def test_average_unequal_rings(C, offs):
    import paper_2401_01728_amd as rv
    n, R = offs[-1], len(offs) - 1
    xs = _replicas(90 + C, C, n)
    g = gen.normal_f32(90 + C, 99, n, std=1e-3)
    dx = [dev(x) for x in xs]
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    rv.cluster_average(dx, R, mean_out=out, grad=dev(g), grad_replica=C - 1, eta=0.5, ring_offsets=offs)
    got = out.cpu().numpy()
    assert np.array_equal(got, average.ring_order_mean_f32(xs, R, g, C - 1, 0.5, ring_offsets=offs))
    ref = average.direct_mean(xs, g, C - 1, 0.5)
    bound = 1e-6 * (np.mean(np.abs(np.stack(xs)).astype(np.float64), axis=0) + 0.5 * np.abs(g) / C)
    assert np.all(np.abs(got.astype(np.float64) - ref) <= bound)
    eq = [(r * n) // 4 for r in range(5)]                          # equal table == default partition
    out2 = torch.empty(n, dtype=torch.float32, device="cuda"); out3 = torch.empty_like(out2)
    rv.cluster_average(dx, 4, mean_out=out2, ring_offsets=eq)
    rv.cluster_average(dx, 4, mean_out=out3)
    assert torch.equal(out2, out3)
    for bad in ([1, n], [0, n - 1], [0, 10, 5, n]):
        with pytest.raises(rv.RvError):
            rv.cluster_average(dx, len(bad) - 1, mean_out=out, ring_offsets=bad)
