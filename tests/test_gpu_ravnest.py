"""The method's outer loop (Alg. 2) through the C ABI: C stages in one HBM, local steps and
periodic ring-partitioned averaging with the sampled peer's step folded in, against the oracle."""
import numpy as np
import pytest
import torch

from oracle import blocks, ravnest as oravnest, stage as ostage
from paper_2401_01728_amd.inputs import gen
from util import bf16_normal, dev, host64, rel_l2
from test_gpu_mlp import kaiming_uniform_flat

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("C,R,kappa", [(3, 2, 3), (4, 4, 1), (2, 1, 4)])
def test_mlp_clusters_follow_alg2(C, R, kappa):
    import paper_2401_01728_amd as rv
    dims, mb, eta, n = [33, 17, 9], 6, 0.05, 13
    w0 = kaiming_uniform_flat(8, dims)
    gs = [rv.Stage.mlp(dims, mb, 0, eta) for _ in range(C)]
    os_ = [ostage.Stage("mlp", 0, eta, w0, dims=dims) for _ in range(C)]
    for g in gs:
        g.set_params(dev(w0))
    picks = [int(v) for v in np.random.default_rng(C).integers(0, C, size=n)]
    mean = w0.astype(np.float64)
    for t, i in enumerate(picks):
        x = gen.normal_f32(8, 10 + t, mb * dims[0]).reshape(mb, dims[0])
        tgt = gen.normal_f32(8, 100 + t, mb * dims[-1]).reshape(mb, dims[-1])
        sync = (t + 1) % kappa == 0
        y = gs[i].forward(t, dev(x))
        yo = os_[i].forward(t, x)
        assert rel_l2(host64(y), yo) < 1e-5
        dy = (2 * (host64(y) - tgt) / tgt.size).astype(np.float32)     # MSE in the harness
        gs[i].defer_update(sync)
        dx = gs[i].backward(t, dev(dy))
        dxo = os_[i].backward(t, dy, defer=sync)
        assert rel_l2(host64(dx), dxo) < 1e-5
        if sync:
            rv.cluster_sync(gs, R, pending=i)
            gs[i].defer_update(False)
            oravnest.cluster_sync(os_, R, pending=i)
            p0 = gs[0].get_params()
            for g in gs[1:]:
                assert torch.equal(g.get_params(), p0)             # one mean, written to all
        mean = mean - (eta / C) * os_[i].last_grad                 # Eq. 17
        got = sum(host64(g.get_params()) for g in gs) / C
        assert rel_l2(got - w0, mean - w0) < 1e-4
    for g, o in zip(gs, os_):
        assert rel_l2(host64(g.get_params()) - w0, o.w - w0) < 1e-4
    with pytest.raises(rv.RvError):
        rv.cluster_sync(gs, R, pending=C)
    with pytest.raises(rv.RvError):
        rv.cluster_sync([gs[0], gs[0]], R)


def test_decoder_clusters_with_microbatches_in_flight():
    """Two decoder stages with staleness 1 inside each: the sync publishes the mean as a new weight
    version while a microbatch forwarded before it is still in flight and is backwarded at the
    version it saw."""
    import paper_2401_01728_amd as rv
    from test_gpu_decoder import decoder_params_host, TOL
    L, d, H, f, S, mb, tau, eta, C, R = 1, 128, 2, 256, 64, 2, 1, 1e-2, 2, 2
    w0 = decoder_params_host(77, L, d, f)
    gs = [rv.Stage.decoder(L, d, H, f, S, mb, tau, eta) for _ in range(C)]
    os_ = [ostage.Stage("decoder", tau, eta, w0, n_blocks=L, d=d, h=H, f=f) for _ in range(C)]
    for g in gs:
        g.set_params(dev(w0))
    x = {}; dy = {}
    for t in range(4):
        x[t] = bf16_normal(77, 1000 + t, (mb, S, d)); dy[t] = bf16_normal(77, 2000 + t, (mb, S, d), std=1e-3)
    # cluster 0: F0 F1 B0(deferred) | sync | B1 at the pre-sync version, then F2 at the mean
    for t in (0, 1):
        assert rel_l2(host64(gs[0].forward(t, x[t][0])), os_[0].forward(t, x[t][1])) < TOL
    gs[0].defer_update(True)
    assert rel_l2(host64(gs[0].backward(0, dy[0][0])), os_[0].backward(0, dy[0][1], defer=True)) < TOL
    gs[0].defer_update(False)
    rv.cluster_sync(gs, R, pending=0); oravnest.cluster_sync(os_, R, pending=0)
    assert torch.equal(gs[0].get_params(), gs[1].get_params())
    assert rel_l2(host64(gs[1].get_params()) - w0, os_[1].w - w0) < TOL
    assert rel_l2(host64(gs[0].backward(1, dy[1][0])), os_[0].backward(1, dy[1][1])) < TOL
    assert os_[0].last_staleness == 1                                  # the sync counted as an update
    for g, o in zip(gs, os_):
        assert rel_l2(host64(g.forward(2, x[2][0])), o.forward(2, x[2][1])) < TOL
        assert rel_l2(host64(g.backward(2, dy[2][0])), o.backward(2, dy[2][1])) < TOL
        assert rel_l2(host64(g.get_params()) - w0, o.w - w0) < TOL
