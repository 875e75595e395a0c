"""Decoder stage vs the oracle: the stage step of paper Alg. 1 with the stale-gradient
update of Eq. 2 (forward(t), backward(t - tau) at the stashed weight version, update).

Both sides receive the same values: fp32 master weights; activations and upstream
gradients already rounded to bf16.  Bars (bf16 products, fp32 accumulation): for outputs,
input gradients and every parameter-gradient tensor 2e-2 normwise AND element by element
|got - ref| <= 2e-2 * (|ref| + rms(ref)) (util.close; achieved errors are printed at the end
of the run); the update itself 1e-6 against w_old - eta * g_gpu in fp64.
"""
import numpy as np
import pytest
import torch

from oracle import blocks, stage as ostage
from paper_2401_01728_amd.inputs import gen
from util import bf16_normal, close, dev, host64, rel_l2

pytestmark = pytest.mark.gpu

TOL = 2e-2


def decoder_params_host(seed, L, d, f):
    """weights, biases, LN beta ~ N(0, 0.02); LN gamma ~ 1 + N(0, 0.02); canonical order."""
    per = 4 * d * d + 2 * d * f + 9 * d + f
    w = gen.normal_f32(seed, 0, L * per, 0.0, 0.02)
    for l in range(L):
        base = l * per
        w[base:base + d] += np.float32(1.0)
        o2 = base + 2 * d + 3 * d * d + 3 * d + d * d + d
        w[o2:o2 + d] += np.float32(1.0)
    return w


def check_tensors(got_flat, ref_flat, shapes, tol=TOL, what="", group=None):
    """Every parameter-gradient tensor on its own (got_flat may be fp32: widened per tensor)."""
    got = blocks.unflatten(got_flat, shapes); ref = blocks.unflatten(ref_flat, shapes)
    grp = group or what.split(" step")[0] + " param grads"
    for name, _ in shapes:
        close(got[name], ref[name], tol, "%s %s" % (what, name), group=grp)


def check_update(w_new, w_old, gg, eta):
    """Eq. 2 in isolation: the new master against w_old - eta * (the GPU's own gradient) in fp64."""
    e = np.float64(np.float32(eta))
    for lo in range(0, w_new.size, 1 << 24):
        sl = slice(lo, lo + (1 << 24))
        wn, wo, g = (np.asarray(a[sl], dtype=np.float64) for a in (w_new, w_old, gg))
        assert np.all(np.abs(wn - (wo - e * g)) <= 1e-6 * (np.abs(wo) + eta * np.abs(g)))


def run_schedule(L, d, H, f, S, mb, tau, n_mb, seed, eta=1e-3, grad_std=1e-3, fused_step=False):
    import paper_2401_01728_amd as rv
    shapes = blocks.decoder_param_shapes(L, d, f)
    w0 = decoder_params_host(seed, L, d, f)
    g = rv.Stage.decoder(L, d, H, f, S, mb, tau, eta, keep_grad=True)
    assert g.num_params == w0.size
    g.set_params(dev(w0))
    o = ostage.Stage("decoder", tau, eta, w0, n_blocks=L, d=d, h=H, f=f)
    tag = "decoder L%d d%d S%d tau%d" % (L, d, S, tau)
    for t in range(n_mb + tau):
        j = t - tau
        both = fused_step and t < n_mb and j >= 0
        if t < n_mb:
            x, x64 = bf16_normal(seed, 1000 + t, (mb, S, d))
        if j >= 0:
            dy, dy64 = bf16_normal(seed, 2000 + j, (mb, S, d), std=grad_std)
            w_old = host64(g.get_params())
        if both:                        # rv_stage_step: the two halves overlap on two streams
            y, dx = g.step(t, x, j, dy)
        if t < n_mb:
            if not both:
                y = g.forward(t, x)
            close(host64(y), o.forward(t, x64), TOL, "out %d" % t, group=tag + " out")
        if j >= 0:
            if not both:
                dx = g.backward(j, dy)
            dxo = o.backward(j, dy64)
            assert o.last_staleness == min(j, tau)
            close(host64(dx), dxo, TOL, "grad_in %d" % j, group=tag + " grad_in")
            gg = host64(g.last_grad())
            check_tensors(gg, o.last_grad, shapes, what="grad step %d" % j, group=tag + " param grads")
            check_update(host64(g.get_params()), w_old, gg, eta)
    assert g.in_flight == 0
    # after n_mb stale updates the two parameter vectors still agree to the gradient bar times eta
    assert rel_l2(host64(g.get_params()) - w0, o.w - w0) < TOL
    return g, o


@pytest.mark.parametrize("L,d,H,f,S,mb,tau", [
    (2, 128, 2, 256, 128, 2, 2),       # dh = 64, several tiles per product
    (1, 256, 2, 512, 192, 1, 1),       # dh = 128, seq not a multiple of 128
    (3, 192, 3, 320, 64, 3, 0),        # tau = 0: sequential SGD; widths that are not multiples of 128
])
def test_small_stage_schedules(L, d, H, f, S, mb, tau):
    run_schedule(L, d, H, f, S, mb, tau, n_mb=2 * tau + 2, seed=20 + L)


@pytest.mark.parametrize("L,d,H,f,S,mb,tau", [(2, 128, 2, 256, 128, 2, 2), (2, 256, 2, 512, 128, 1, 0),
                                               (3, 192, 3, 320, 64, 3, 1)])
def test_fused_step_equals_forward_then_backward(L, d, H, f, S, mb, tau):
    """rv_stage_step must give what forward(t); backward(t - tau) gives (oracle order F, B)."""
    run_schedule(L, d, H, f, S, mb, tau, n_mb=2 * tau + 4, seed=40 + L, fused_step=True)


def test_fused_step_is_bitwise_the_two_calls():
    """... and the update applied inside the gradient kernels (the default) gives, bit for bit, the
    parameters of the variant that also keeps the gradient; only the latter can be read back."""
    import paper_2401_01728_amd as rv
    L, d, H, f, S, mb, tau = 2, 128, 2, 256, 128, 2, 2
    w0 = dev(decoder_params_host(9, L, d, f))
    res = []
    for fused, keep in ((False, False), (True, False), (True, True)):
        g = rv.Stage.decoder(L, d, H, f, S, mb, tau, 1e-3, keep_grad=keep); g.set_params(w0)
        outs = []
        for t in range(8 + tau):
            j = t - tau
            x, _ = bf16_normal(9, 1000 + t, (mb, S, d)); dy, _ = bf16_normal(9, 2000 + max(j, 0), (mb, S, d), std=1e-3)
            if fused and t < 8 and j >= 0:
                y, dx = g.step(t, x, j, dy); outs += [y, dx]
            else:
                if t < 8:
                    outs.append(g.forward(t, x))
                if j >= 0:
                    outs.append(g.backward(j, dy))
        outs.append(g.get_params())
        torch.cuda.synchronize()
        res.append([o.clone() for o in outs])
        if keep:
            assert torch.isfinite(g.last_grad()).all()
        else:
            with pytest.raises(rv.RvError):
                g.last_grad()
    for other in res[1:]:
        assert len(other) == len(res[0])
        for a, b in zip(res[0], other):
            assert torch.equal(a, b)


def test_deep_staleness_reduced_shape():
    """The deep-staleness stage's whole run of 64 interleaved microbatches (4 warm-up forwards, 60
    steady steps through rv_stage_step, 4 draining backwards; 12 blocks, tau = 4, 5 stash slots
    and weight versions) at reduced widths: d = 448 with 7 heads of 64 (1600 / 4 = 400 is not a
    multiple of the head size), ffn 1792, seq 128, microbatch 2."""
    run_schedule(12, 448, 7, 1792, 128, 2, 4, n_mb=64, seed=5, fused_step=True)


def test_backward_uses_the_stashed_version_not_the_current_one():
    """With the configs' learning rate one update moves a weight by less than bf16 resolves, so a
    backward at the wrong version would pass every other test.  Here eta is chosen so that one
    update displaces the parameters by about 10 % of their norm: the stage must still match the
    oracle, and an oracle with the mistake planted in it (backward at the CURRENT parameters)
    must be far outside the bar, else this test could not tell the difference."""
    import paper_2401_01728_amd as rv
    L, d, H, f, S, mb, tau, seed, n = 2, 128, 2, 256, 128, 2, 2, 77, 5
    shapes = blocks.decoder_param_shapes(L, d, f)
    w0 = decoder_params_host(seed, L, d, f)
    xs = [bf16_normal(seed, 1000 + t, (mb, S, d)) for t in range(n)]
    dys = [bf16_normal(seed, 2000 + t, (mb, S, d), std=1e-3) for t in range(n)]
    _, g0 = blocks.decoder_backward(w0.astype(np.float64), L, d, H, f, 1e-5, xs[0][1], dys[0][1])
    eta = float(np.float32(0.1 * np.linalg.norm(w0) / np.linalg.norm(g0)))

    class CurrentWeightsStage(ostage.Stage):           # the planted mistake
        def backward(self, mb_id, dy, defer=False):
            _, x, k = self.live[mb_id]
            self.live[mb_id] = (self.w.copy(), x, k)
            return super().backward(mb_id, dy, defer)

    g = rv.Stage.decoder(L, d, H, f, S, mb, tau, eta, keep_grad=True); g.set_params(dev(w0))
    o = ostage.Stage("decoder", tau, eta, w0, n_blocks=L, d=d, h=H, f=f)
    bad = CurrentWeightsStage("decoder", tau, eta, w0, n_blocks=L, d=d, h=H, f=f)
    told_apart = 0.0
    for t in range(n + tau):
        j = t - tau
        if t < n and j >= 0:
            y, dx = g.step(t, xs[t][0], j, dys[j][0])
        elif t < n:
            y = g.forward(t, xs[t][0])
        else:
            dx = g.backward(j, dys[j][0])
        if t < n:
            close(host64(y), o.forward(t, xs[t][1]), TOL, "out %d" % t, group="large-step stage out")
            bad.forward(t, xs[t][1])
        if j >= 0:
            close(host64(dx), o.backward(j, dys[j][1]), TOL, "grad_in %d" % j, group="large-step stage grad_in")
            check_tensors(host64(g.last_grad()), o.last_grad, shapes, what="grad step %d" % j,
                          group="large-step stage param grads")
            bad.backward(j, dys[j][1])
            if o.last_staleness > 0:
                told_apart = max(told_apart, rel_l2(bad.last_grad, o.last_grad))
    assert told_apart > 5 * TOL, told_apart


def test_decoder_error_paths():
    import paper_2401_01728_amd as rv
    with pytest.raises(rv.RvError):
        rv.Stage.decoder(1, 100, 1, 256, 64, 1, 0, 1e-3)          # d % 64
    with pytest.raises(rv.RvError):
        rv.Stage.decoder(1, 192, 2, 256, 64, 1, 0, 1e-3)          # head size 96
    with pytest.raises(rv.RvError):
        rv.Stage.decoder(1, 128, 2, 256, 100, 1, 0, 1e-3)         # seq % 64
    g = rv.Stage.decoder(1, 128, 2, 256, 64, 1, 1, 1e-3)
    x = torch.zeros(1, 64, 128, dtype=torch.bfloat16, device="cuda")
    g.forward(0, x); g.forward(1, x)
    with pytest.raises(rv.RvError) as e:
        g.forward(2, x)
    assert e.value.status == rv.api.RV_E_STASH_FULL
    with pytest.raises(rv.RvError) as e:
        g.backward(5, x)
    assert e.value.status == rv.api.RV_E_UNKNOWN_MB
    g.backward(1, x); g.backward(0, x)
    assert g.in_flight == 0


@pytest.mark.parametrize("A,momentum,wd", [(2, 0.0, 0.0), (1, 0.9, 5e-4), (2, 0.9, 5e-4)])
def test_decoder_stage_with_accumulation_in_fused_steps(A, momentum, wd):
    """Gradient accumulation (section 4.2) and the momentum / weight-decay optimiser (section 4.1)
    through rv_stage_step: block-wise accumulate / update on the side stream, forwards bound to
    a version that only every A-th backward replaces."""
    import paper_2401_01728_amd as rv
    L, d, H, f, S, mb, tau, eta = 2, 128, 2, 256, 128, 2, 2, 1e-2
    shapes = blocks.decoder_param_shapes(L, d, f)
    w0 = decoder_params_host(31, L, d, f)
    g = rv.Stage.decoder(L, d, H, f, S, mb, tau, eta); g.set_params(dev(w0)); g.set_accumulation(A)
    if momentum or wd:
        g.set_optimizer(momentum, wd)
    o = ostage.Stage("decoder", tau, eta, w0, n_blocks=L, d=d, h=H, f=f, accumulate=A, momentum=momentum,
                     weight_decay=wd)
    n = 7
    for t in range(n + tau):
        j = t - tau
        if t < n:
            x, x64 = bf16_normal(31, 1000 + t, (mb, S, d))
        if j >= 0:
            dy, dy64 = bf16_normal(31, 2000 + j, (mb, S, d), std=1e-3)
        if t < n and j >= 0:
            y, dx = g.step(t, x, j, dy)
        elif t < n:
            y = g.forward(t, x)
        else:
            dx = g.backward(j, dy)
        tag = "decoder accumulate"
        if t < n:
            close(host64(y), o.forward(t, x64), TOL, "out %d" % t, group=tag + " out")
        if j >= 0:
            close(host64(dx), o.backward(j, dy64), TOL, "grad_in %d" % j, group=tag + " grad_in")
            check_tensors(host64(g.last_grad()), o.last_grad, shapes, what="grad step %d" % j, group=tag + " param grads")
    assert o.k == n // A
    assert rel_l2(host64(g.get_params()) - w0, o.w - w0) < TOL
