"""Parity at the benchmark shapes, in the launch configuration bench.py times.

config 2 (4 blocks, d 1024, seq 512, microbatch 8): one whole stage step against the
oracle - out, grad_in, every parameter-gradient tensor, the update.
configs 3 and 5 (d 2048 x 8 blocks; d 1600, 25 heads x 12 blocks): the GPU runs the full
microbatch; sequences are independent in the forward and in the input gradient, so the
oracle computes ONE sequence and that slice of out / grad_in is compared (a full fp64 step
would take the host tens of minutes).  Parameter gradients at these two shapes are covered
by the reduced-shape schedules in test_gpu_decoder.py.
config 4 (N = 1e9, C = 16, folded gradient, R in {1,2,4,8}): windows around every ring and
chunk boundary plus random indices, regenerated on the host from the counter generator,
bit-exact against the fp32 ring-order twin and within the 1e-6 bound of the fp64 mean.
"""
import numpy as np
import pytest
import torch

from oracle import average, blocks, stage as ostage
from paper_2401_01728_amd.inputs import gen
from util import bf16_normal, dev, host64, rel_l2
from test_gpu_decoder import TOL, check_tensors, decoder_params_host

pytestmark = pytest.mark.gpu


def test_config2_full_stage_step():
    import paper_2401_01728_amd as rv
    L, d, H, f, S, mb, tau, eta = 4, 1024, 16, 4096, 512, 8, 2, 1e-3
    shapes = blocks.decoder_param_shapes(L, d, f)
    w0 = decoder_params_host(2, L, d, f)
    assert w0.size == 50384896
    g = rv.Stage.decoder(L, d, H, f, S, mb, tau, eta); g.set_params(dev(w0))
    o = ostage.Stage("decoder", tau, eta, w0, n_blocks=L, d=d, h=H, f=f)
    x, x64 = bf16_normal(2, 1000, (mb, S, d))
    dy, dy64 = bf16_normal(2, 2000, (mb, S, d), std=1e-3)
    y = g.forward(0, x)
    assert rel_l2(host64(y), o.forward(0, x64)) < TOL
    dx = g.backward(0, dy)
    dxo = o.backward(0, dy64)
    assert rel_l2(host64(dx), dxo) < TOL
    gg = host64(g.last_grad())
    check_tensors(gg, o.last_grad, shapes, what="config 2")
    w_new = host64(g.get_params())
    assert np.all(np.abs(w_new - (w0.astype(np.float64) - np.float64(np.float32(eta)) * gg))
                  <= 1e-6 * (np.abs(w0) + eta * np.abs(gg)))


@pytest.mark.parametrize("name,L,d,H,f,S,mb,tau", [("config3", 8, 2048, 16, 8192, 1024, 4, 3),
                                                    ("config5", 12, 1600, 25, 6400, 1024, 8, 4)])
def test_large_stage_one_sequence(name, L, d, H, f, S, mb, tau):
    import paper_2401_01728_amd as rv
    from paper_2401_01728_amd.inputs import device
    seed = 3 if name == "config3" else 5
    per = 4 * d * d + 2 * d * f + 9 * d + f
    w = torch.empty(L * per, dtype=torch.float32, device="cuda")
    device.fill_normal_(w, seed, 0, 0.0, 0.02)            # same recipe as decoder_params_host, on the device
    for l in range(L):
        w[l * per:l * per + d] += 1.0
        o2 = l * per + 2 * d + 3 * d * d + 3 * d + d * d + d
        w[o2:o2 + d] += 1.0
    g = rv.Stage.decoder(L, d, H, f, S, mb, tau, 1e-3); g.set_params(w)
    x, x64 = bf16_normal(seed, 1000, (mb, S, d))
    dy, dy64 = bf16_normal(seed, 2000, (mb, S, d), std=1e-3)
    # the fused step needs tau microbatches in flight first; use the plain calls here and the
    # fused call for a second microbatch so both launch paths run at this shape
    y = g.forward(0, x)
    y1, dx = g.step(1, x, 0, dy)
    b = 1
    o = ostage.Stage("decoder", 0, 1e-3, w.cpu().numpy(), n_blocks=L, d=d, h=H, f=f)
    yo = o.forward(0, x64[b:b + 1])
    assert rel_l2(host64(y[b:b + 1]), yo) < TOL
    assert rel_l2(host64(y1[b:b + 1]), yo) < TOL          # forward(1) ran before the update: same weights
    dxo = o.backward(0, dy64[b:b + 1])
    assert rel_l2(host64(dx[b:b + 1]), dxo) < TOL


@pytest.mark.parametrize("R", [1, 2, 4, 8])
def test_config4_sampled(R):
    import paper_2401_01728_amd as rv
    from paper_2401_01728_amd.inputs import device
    n, C, eta, seed, gr = 1_000_000_000, 16, 1e-3, 4, 0
    if torch.cuda.get_device_properties(0).total_memory < 90e9:
        pytest.skip("needs 72 GB of device memory")
    shared = device.fill_normal_(torch.empty(n, dtype=torch.float32, device="cuda"), seed, 0)
    reps = []
    for c in range(C):
        r = device.fill_normal_(torch.empty(n, dtype=torch.float32, device="cuda"), seed, 1 + c)
        r += shared
        reps.append(r)
    del shared
    grad = device.fill_normal_(torch.empty(n, dtype=torch.float32, device="cuda"), seed, 99, 0.0, 1e-3)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    rv.cluster_average(reps, R, mean_out=out, grad=grad, grad_replica=gr, eta=eta)
    torch.cuda.synchronize()
    # sample: +-40 elements around every chunk boundary, the two ends, 1e6 random indices
    bounds = average.ring_partition(n, R, C)
    idx = [np.arange(0, 4096), np.arange(n - 4096, n)]
    for rb in bounds:
        for e in rb[1:]:
            idx.append(np.arange(max(e - 40, 0), min(e + 40, n)))
    idx.append(np.random.default_rng(R).integers(0, n, size=1_000_000))
    idx = np.unique(np.concatenate(idx)).astype(np.uint64)
    o = gen.normal_f32_at(seed, 0, idx)
    xs = [(o + gen.normal_f32_at(seed, 1 + c, idx)).astype(np.float32) for c in range(C)]
    gh = gen.normal_f32_at(seed, 99, idx, 0.0, 1e-3)
    got = out[torch.from_numpy(idx.astype(np.int64)).cuda()].cpu().numpy()
    # owning chunk of every sampled index -> rotation of the ring-order sum
    j_of = np.empty(idx.size, dtype=np.int64)
    for rb in bounds:
        for j in range(C):
            m = (idx >= rb[j]) & (idx < rb[j + 1])
            j_of[m] = j
    step = gh * np.float32(eta)
    xs[gr] = xs[gr] - step
    X = np.stack(xs)                                      # [C, m] fp32
    acc = X[j_of % C, np.arange(idx.size)].copy()
    for s in range(1, C):
        acc = acc + X[(j_of + s) % C, np.arange(idx.size)]
    twin = acc / np.float32(C)
    assert np.array_equal(got.view(np.uint32), twin.astype(np.float32).view(np.uint32))
    ref = X.astype(np.float64).mean(axis=0)               # xs[gr] already holds the folded step (fp32 inputs)
    bound = 1e-6 * (np.abs(X).astype(np.float64).mean(axis=0) + eta * np.abs(gh) / C)
    assert np.all(np.abs(got.astype(np.float64) - ref) <= bound + 1e-6 * np.abs(step) / C)


@pytest.mark.parametrize("name,L,d,H,f,S,mb,tau", [("config2", 4, 1024, 16, 4096, 512, 8, 2),
                                                   ("config5 (4 of 12 blocks)", 4, 1600, 25, 6400, 1024, 8, 4)])
def test_fused_steps_at_bench_shapes_are_bitwise_the_sequential_calls(name, L, d, H, f, S, mb, tau):
    """rv_stage_step as bench.py times it (forward, backward chain and parameter-gradient work on
    three streams, buffers alternating between blocks) must give, bit for bit, what the same
    schedule gives as forward(t); backward(t - tau) on one stream - at the real shapes, where a
    missing dependency between the streams would show."""
    import paper_2401_01728_amd as rv
    from paper_2401_01728_amd.inputs import device
    w0 = dev(decoder_params_host(2, L, d, f))
    n = tau + 5
    xs = [device.fill_normal_(torch.empty(mb, S, d, dtype=torch.bfloat16, device="cuda"), 2, 1000 + t) for t in range(n)]
    dys = [device.fill_normal_(torch.empty(mb, S, d, dtype=torch.bfloat16, device="cuda"), 2, 2000 + t, 0.0, 1e-3)
           for t in range(n)]
    res = []
    for fused in (False, True):
        g = rv.Stage.decoder(L, d, H, f, S, mb, tau, 1e-3); g.set_params(w0)
        outs = []
        for t in range(n + tau):
            j = t - tau
            if fused and t < n and j >= 0:
                y, dx = g.step(t, xs[t], j, dys[j]); outs += [y.clone(), dx.clone()]
            else:
                if t < n:
                    outs.append(g.forward(t, xs[t]).clone())
                if j >= 0:
                    outs.append(g.backward(j, dys[j]).clone())
        outs.append(g.get_params().clone()); outs.append(g.last_grad().clone())
        torch.cuda.synchronize()
        res.append(outs)
        del g
    assert len(res[0]) == len(res[1])
    for k, (a, b) in enumerate(zip(*res)):
        assert torch.equal(a, b), (name, k)
