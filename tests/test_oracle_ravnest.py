"""Pins of the Alg. 2 oracle (oracle/ravnest.py) by facts that do not come from it."""
import numpy as np

from oracle import blocks, ravnest, stage

DIMS = [4, 6, 3]
P = 4 * 6 + 6 + 6 * 3 + 3


def _stages(C, eta, w0):
    return [stage.Stage("mlp", 0, eta, w0, dims=DIMS) for _ in range(C)]


def _batches(seed, n):
    rng = np.random.default_rng(seed)
    xs = [rng.normal(size=(5, 4)) for _ in range(n)]
    ts = [rng.normal(size=(5, 3)) for _ in range(n)]
    return xs, ts, (lambda t, i: (xs[t], lambda y: 2 * (y - ts[t]) / y.size))


def test_one_cluster_is_plain_sgd_whatever_kappa():
    """C = 1: the mean of one replica with its pending step folded in IS the step."""
    rng = np.random.default_rng(0)
    w0 = rng.normal(size=P) * 0.5
    xs, ts, fn = _batches(1, 9)
    for kappa in (1, 2, 4):
        st = _stages(1, 0.05, w0)
        ravnest.run(st, [0] * 9, kappa, 2, fn)
        w = w0.copy()
        for t in range(9):
            y = blocks.mlp_forward(w, DIMS, xs[t])
            _, g = blocks.mlp_backward(w, DIMS, xs[t], 2 * (y - ts[t]) / y.size)
            w = w - 0.05 * g
        assert np.allclose(st[0].w, w, rtol=0, atol=1e-14)


def test_kappa_one_is_single_model_sgd_with_step_eta_over_C():
    """kappa = 1: every step is an all-reduce, the replicas never part, and by Eq. 17 the common
    vector moves by -(eta/C) g with g taken at the common vector."""
    rng = np.random.default_rng(2)
    w0 = rng.normal(size=P) * 0.5
    C, eta, n = 3, 0.06, 7
    xs, ts, fn = _batches(3, n)
    st = _stages(C, eta, w0)
    picks = [int(v) for v in rng.integers(0, C, size=n)]
    ravnest.run(st, picks, 1, 2, fn)
    w = w0.copy()
    for t in range(n):
        y = blocks.mlp_forward(w, DIMS, xs[t])
        _, g = blocks.mlp_backward(w, DIMS, xs[t], 2 * (y - ts[t]) / y.size)
        w = w - (eta / C) * g
    for s in st:
        assert np.allclose(s.w, w, rtol=0, atol=1e-13)


def test_mean_follows_eq17_and_replicas_agree_after_each_sync():
    rng = np.random.default_rng(4)
    w0 = rng.normal(size=P) * 0.5
    C, eta, kappa, n = 4, 0.05, 3, 12
    xs, ts, fn = _batches(5, n)
    st = _stages(C, eta, w0)
    picks = [int(v) for v in rng.integers(0, C, size=n)]
    mean = w0.copy()
    for t, i in enumerate(picks):
        before = [s.w.copy() for s in st]
        x, dy_fn = fn(t, i)
        y = st[i].forward(t, x)
        sync = (t + 1) % kappa == 0
        st[i].backward(t, dy_fn(y), defer=sync)
        g = st[i].last_grad
        if sync:
            rounds = ravnest.cluster_sync(st, 2, pending=i)
            assert rounds == 2 * (C - 1)
            for s in st[1:]:
                assert np.array_equal(s.w, st[0].w)
        else:
            for j, s in enumerate(st):
                if j != i:
                    assert np.array_equal(s.w, before[j])        # only the sampled peer moves (Eq. 3)
        mean = mean - (eta / C) * g                                # Eq. 17 holds at every step
        assert np.allclose(sum(s.w for s in st) / C, mean, rtol=0, atol=1e-13)


def test_deferred_backward_leaves_parameters_and_counts_no_update():
    rng = np.random.default_rng(6)
    w0 = rng.normal(size=P) * 0.5
    s = stage.Stage("mlp", 0, 0.05, w0, dims=DIMS)
    x = rng.normal(size=(5, 4)); dy = rng.normal(size=(5, 3))
    s.forward(0, x); s.backward(0, dy, defer=True)
    assert np.array_equal(s.w, w0) and s.k == 0
    _, g = blocks.mlp_backward(w0, DIMS, x, dy)
    assert np.array_equal(s.last_grad, g)
    s.install(w0 - 1.0)
    assert s.k == 1
