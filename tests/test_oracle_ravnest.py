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


# ---- clusters that are chains of peers ---------------------------------------------------------
CH = [[4, 6, 3], [3, 5, 2]]                       # two peers per cluster: 4 -> 6 -> 3 | 3 -> 5 -> 2
CHP = [blocks.num_params(blocks.mlp_param_shapes(d)) for d in CH]


def _chains(C, eta, w0s):
    return [[stage.Stage("mlp", 0, eta, w0s[p], dims=CH[p]) for p in range(2)] for _ in range(C)]


def _chain_batches(seed, n):
    rng = np.random.default_rng(seed)
    xs = [rng.normal(size=(5, 4)) for _ in range(n)]
    ts = [rng.normal(size=(5, 2)) for _ in range(n)]
    return xs, ts, (lambda m, i: (xs[m], lambda y: 2 * (y - ts[m]) / y.size))


def _composite_grads(w0, w1, x, t):
    """Gradient of the loss of the composed model by its definition: both peers' forward, then the
    chain rule through the second peer into the first - coded here, not taken from ravnest.py."""
    h = blocks.mlp_forward(w0, CH[0], x)
    y = blocks.mlp_forward(w1, CH[1], h)
    dh, g1 = blocks.mlp_backward(w1, CH[1], h, 2 * (y - t) / y.size)
    _, g0 = blocks.mlp_backward(w0, CH[0], x, dh)
    return g0, g1


def test_one_chain_is_block_sgd_on_the_composed_model():
    """C = 1, any kappa: the last peer steps first, the first peer's gradient is taken through the
    last peer's parameters as they were in the forward (Eq. 2) - a separately written loop."""
    rng = np.random.default_rng(11)
    w0s = [rng.normal(size=n) * 0.5 for n in CHP]
    xs, ts, fn = _chain_batches(12, 8)
    for kappa in (1, 3, 5):
        cl = _chains(1, 0.05, w0s)
        ravnest.run_chains(cl, [0] * 8, kappa, 2, fn)
        a, b = w0s[0].copy(), w0s[1].copy()
        for m in range(8):
            g0, g1 = _composite_grads(a, b, xs[m], ts[m])
            a, b = a - 0.05 * g0, b - 0.05 * g1
        assert np.allclose(cl[0][0].w, a, rtol=0, atol=1e-13)
        assert np.allclose(cl[0][1].w, b, rtol=0, atol=1e-13)


def test_chains_over_many_iterations_follow_eq17_block_by_block():
    """120 peer iterations over 4 clusters of 2 peers, kappa = 7: at every iteration the mean of a
    peer position over the clusters moves by -(eta/C) g on the block of the peer that ran and not
    at all on the other block (Eq. 4, Eq. 17); after an averaging iteration all clusters agree on
    every block; between them only the sampled peer moves."""
    rng = np.random.default_rng(13)
    C, eta, kappa, n = 4, 0.04, 7, 60
    w0s = [rng.normal(size=k) * 0.5 for k in CHP]
    xs, ts, fn = _chain_batches(14, n)
    cl = _chains(C, eta, w0s)
    picks = [int(v) for v in rng.integers(0, C, size=n)]
    means = [w.copy() for w in w0s]
    seen = {"t": 0, "syncs": 0}
    before = {}

    def snapshot():
        for c in range(C):
            for p in range(2):
                before[(c, p)] = cl[c][p].w.copy()

    def on_event(t, i, p, sync):
        assert t == seen["t"]
        seen["t"] += 1
        seen["syncs"] += int(sync)
        means[p] = means[p] - (eta / C) * cl[i][p].last_grad
        for q in range(2):
            got = sum(cl[c][q].w for c in range(C)) / C
            assert np.allclose(got, means[q], rtol=0, atol=1e-12)
        if sync:
            for q in range(2):
                for c in range(1, C):
                    assert np.array_equal(cl[c][q].w, cl[0][q].w)
        else:
            for c in range(C):
                for q in range(2):
                    if (c, q) != (i, p):
                        assert np.array_equal(cl[c][q].w, before[(c, q)])
        snapshot()

    snapshot()
    ravnest.run_chains(cl, picks, kappa, 3, fn, on_event)
    assert seen["t"] == 2 * n == 120 and seen["syncs"] == 120 // kappa


def test_state_averaging_takes_the_mean_of_the_momentum_buffers():
    rng = np.random.default_rng(15)
    C, eta = 3, 0.05
    w0 = rng.normal(size=P) * 0.5
    st = [stage.Stage("mlp", 0, eta, w0, dims=DIMS, momentum=0.9, weight_decay=1e-3) for _ in range(C)]
    for t in range(4):                                            # local steps part the clusters
        for i, s in enumerate(st):
            x = rng.normal(size=(5, 4)); dy = rng.normal(size=(5, 3))
            s.forward(t, x); s.backward(t, dy)
    vbar = sum(s.v for s in st) / C; wbar = sum(s.w for s in st) / C
    ravnest.cluster_sync(st, 2, average_state=True)
    for s in st:
        assert np.allclose(s.v, vbar, rtol=0, atol=1e-15) and np.allclose(s.w, wbar, rtol=0, atol=1e-15)
    # without the flag the buffers are left alone
    v_keep = [s.v.copy() for s in st]
    ravnest.cluster_sync(st, 2)
    assert all(np.array_equal(s.v, v) for s, v in zip(st, v_keep))
