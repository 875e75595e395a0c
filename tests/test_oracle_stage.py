"""Pins for oracle/stage.py: delayed-update semantics (paper Eq. 2, Alg. 1)."""
import numpy as np
import pytest

from oracle import blocks, stage


def _mlp_stage(tau, eta, seed=0, dims=(4, 6, 3)):
    rng = np.random.default_rng(seed)
    P = blocks.num_params(blocks.mlp_param_shapes(list(dims)))
    return stage.Stage("mlp", tau, eta, rng.normal(size=P) * 0.5, dims=list(dims))


def _run_schedule(st, xs, dys_fn, tau):
    """F(t), B(t - tau) interleaved; dys_fn(t, y) gives the upstream gradient."""
    ys = {}
    n = len(xs)
    for t in range(n + tau):
        if t < n:
            ys[t] = st.forward(t, xs[t])
        j = t - tau
        if j >= 0:
            st.backward(j, dys_fn(j, ys[j]))


def test_tau0_is_sequential_sgd_bitwise():
    rng = np.random.default_rng(10)
    dims = [4, 6, 3]
    st = _mlp_stage(0, 0.05)
    w = st.w.copy()
    xs = [rng.normal(size=(5, 4)) for _ in range(6)]
    ts = [rng.normal(size=(5, 3)) for _ in range(6)]
    _run_schedule(st, xs, lambda j, y: 2 * (y - ts[j]) / y.size, 0)
    # separately written plain SGD loop
    for x, t in zip(xs, ts):
        y = blocks.mlp_forward(w, dims, x)
        _, g = blocks.mlp_backward(w, dims, x, 2 * (y - t) / y.size)
        w = w - 0.05 * g
    assert np.array_equal(st.w, w)


def test_scalar_recurrence_hand_values():
    """Linear 1->1 with x = 1, loss y^2/2: s = w + b obeys
    s[k+1] = s[k] - 2*eta*s[max(k - tau, 0)].  eta = 0.1, tau = 2, s0 = 1 gives
    1, .8, .6, .4, .24, .12, .04 (worked by hand)."""
    st = stage.Stage("mlp", 2, 0.1, np.array([0.75, 0.25]), dims=[1, 1])
    seen = [st.w.sum()]
    ys = {}
    n = 6
    for t in range(n + 2):
        if t < n:
            ys[t] = st.forward(t, np.array([[1.0]]))
        if t - 2 >= 0:
            st.backward(t - 2, ys[t - 2])
            seen.append(st.w.sum())
    assert np.allclose(seen, [1.0, 0.8, 0.6, 0.4, 0.24, 0.12, 0.04], atol=1e-15)


@pytest.mark.parametrize("tau", [1, 3])
def test_against_full_weight_history(tau):
    """Brute force: keep every parameter state, recompute each gradient from w[max(k-tau,0)]."""
    rng = np.random.default_rng(11)
    dims = [4, 6, 3]
    st = _mlp_stage(tau, 0.05, seed=3)
    hist = [st.w.copy()]
    xs = [rng.normal(size=(5, 4)) for _ in range(8)]
    dys = [rng.normal(size=(5, 3)) for _ in range(8)]
    stal = []
    ys = {}
    for t in range(8 + tau):
        if t < 8:
            ys[t] = st.forward(t, xs[t])
            assert len(st.live) <= tau + 1
        if t - tau >= 0:
            st.backward(t - tau, dys[t - tau]); stal.append(st.last_staleness)
    for k in range(8):
        wk = hist[max(k - tau, 0)]
        _, g = blocks.mlp_backward(wk, dims, xs[k], dys[k])
        hist.append(hist[-1] - 0.05 * g)
        assert np.array_equal(ys[k], blocks.mlp_forward(wk, dims, xs[k]))
    assert np.array_equal(st.w, hist[-1])
    assert stal == [min(k, tau) for k in range(8)]


def test_stash_accounting_and_errors():
    st = _mlp_stage(2, 0.1)
    x = np.zeros((1, 4))
    for t in range(3):
        st.forward(t, x)
    w = st.w.copy()
    with pytest.raises(stage.StashFull):
        st.forward(3, x)
    with pytest.raises(stage.DuplicateMicrobatch):
        st.forward(1, x)
    with pytest.raises(stage.UnknownMicrobatch):
        st.backward(7, np.zeros((1, 3)))
    assert np.array_equal(st.w, w) and len(st.live) == 3


def test_block_structure_only_own_block_moves():
    a, b = _mlp_stage(0, 0.1, seed=1), _mlp_stage(0, 0.1, seed=2)
    wb = b.w.copy(); wa = a.w.copy()
    a.forward(0, np.ones((2, 4))); a.backward(0, np.ones((2, 3)))
    assert np.array_equal(b.w, wb) and not np.array_equal(a.w, wa)


def test_decoder_stage_uses_forward_time_weights():
    rng = np.random.default_rng(12)
    L, d, h, f = 1, 8, 2, 16
    P = blocks.num_params(blocks.decoder_param_shapes(L, d, f))
    w0 = rng.normal(size=P) * 0.3
    st = stage.Stage("decoder", 1, 0.1, w0, n_blocks=L, d=d, h=h, f=f)
    x0, x1 = rng.normal(size=(1, 3, d)), rng.normal(size=(1, 3, d))
    dy0, dy1 = rng.normal(size=(1, 3, d)), rng.normal(size=(1, 3, d))
    st.forward(0, x0); st.forward(1, x1)
    st.backward(0, dy0)
    dx1 = st.backward(1, dy1)                   # one update happened since forward(1)
    ref_dx1, g1 = blocks.decoder_backward(w0, L, d, h, f, 1e-5, x1, dy1)
    _, g0 = blocks.decoder_backward(w0, L, d, h, f, 1e-5, x0, dy0)
    assert np.array_equal(dx1, ref_dx1) and st.last_staleness == 1
    assert np.allclose(st.w, w0 - 0.1 * g0 - 0.1 * g1, rtol=0, atol=1e-15)


def test_momentum_weight_decay_closed_forms():
    """Linear 1->1, x = 1, upstream gradient fixed at 1: dL/dw = dL/db = 1 every step."""
    eta, mu, wd, n = 0.1, 0.9, 0.0, 6
    st = stage.Stage("mlp", 0, eta, np.array([2.0, 1.0]), dims=[1, 1], momentum=mu, weight_decay=wd)
    for t in range(n):
        st.forward(t, np.array([[1.0]])); st.backward(t, np.array([[1.0]]))
    # v_k = (1 - mu^k)/(1 - mu);  w_n = w_0 - eta * sum_{k=1..n} v_k
    tot = sum((1 - mu ** k) / (1 - mu) for k in range(1, n + 1))
    assert np.allclose(st.w, np.array([2.0, 1.0]) - eta * tot, rtol=0, atol=1e-14)
    # weight decay alone with zero gradient: geometric shrink w_k = w_0 (1 - eta wd)^k
    st = stage.Stage("mlp", 0, 0.1, np.array([2.0, -1.0]), dims=[1, 1], momentum=0.0, weight_decay=0.5)
    for t in range(5):
        st.forward(t, np.array([[0.0]])); st.backward(t, np.array([[0.0]]))
    assert np.allclose(st.w, np.array([2.0, -1.0]) * (1 - 0.05) ** 5, rtol=0, atol=1e-15)
    # both zero: the plain step of Eq. 2, bit for bit
    a, b = _mlp_stage(1, 0.05, seed=4), _mlp_stage(1, 0.05, seed=4)
    b.momentum = b.weight_decay = 0.0
    rng = np.random.default_rng(0)
    xs = [rng.normal(size=(5, 4)) for _ in range(4)]
    _run_schedule(a, xs, lambda j, y: y, 1); _run_schedule(b, xs, lambda j, y: y, 1)
    assert np.array_equal(a.w, b.w)


def test_momentum_against_separate_loop():
    rng = np.random.default_rng(21)
    dims, eta, mu, wd = [4, 6, 3], 0.05, 0.9, 5e-4
    st = stage.Stage("mlp", 0, eta, rng.normal(size=51) * 0.5, dims=dims, momentum=mu, weight_decay=wd)
    w = st.w.copy(); v = np.zeros_like(w)
    for t in range(5):
        x = rng.normal(size=(5, 4)); dy = rng.normal(size=(5, 3))
        st.forward(t, x); st.backward(t, dy)
        _, g = blocks.mlp_backward(w, dims, x, dy)
        v = mu * v + (g + wd * w); w = w - eta * v
    assert np.allclose(st.w, w, rtol=0, atol=1e-15)


def test_accumulation_equals_one_backward_on_the_stacked_batch():
    """Section 4.2: gradients of A microbatches are summed before one update.  With no update in
    between, A microbatches see the same weights, so the sum of their gradients is the gradient
    of the stacked batch (the layers act row by row) - computed here by a stage that never
    accumulates."""
    rng = np.random.default_rng(5)
    dims, eta = [4, 6, 3], 0.05
    w0 = rng.normal(size=51) * 0.5
    xs = [rng.normal(size=(5, 4)) for _ in range(3)]
    dys = [rng.normal(size=(5, 3)) for _ in range(3)]
    a = stage.Stage("mlp", 0, eta, w0, dims=dims, accumulate=3)
    for t in range(3):
        a.forward(t, xs[t])
        assert np.array_equal(a.w, w0)                      # nothing moves before the third backward
        a.backward(t, dys[t])
    b = stage.Stage("mlp", 0, eta, w0, dims=dims)
    b.forward(0, np.concatenate(xs)); b.backward(0, np.concatenate(dys))
    assert np.allclose(a.w, b.w, rtol=0, atol=1e-14)
    assert a.k == 1 and a.n_sum == 0


def test_accumulation_with_staleness_against_separate_loop():
    rng = np.random.default_rng(6)
    dims, eta, tau, A, n = [4, 6, 3], 0.05, 1, 2, 8
    w0 = rng.normal(size=51) * 0.5
    st = stage.Stage("mlp", tau, eta, w0, dims=dims, accumulate=A)
    xs = [rng.normal(size=(5, 4)) for _ in range(n)]
    dys = [rng.normal(size=(5, 3)) for _ in range(n)]
    w = w0.copy(); seen = {}; acc = np.zeros_like(w); cnt = 0; stal = []
    updates = 0; fwd_k = {}
    for t in range(n + tau):
        if t < n:
            st.forward(t, xs[t]); seen[t] = w.copy(); fwd_k[t] = updates
        j = t - tau
        if j >= 0:
            st.backward(j, dys[j]); stal.append(st.last_staleness)
            _, g = blocks.mlp_backward(seen.pop(j), dims, xs[j], dys[j])
            assert stal[-1] == updates - fwd_k[j]
            acc += g; cnt += 1
            if cnt == A:
                w = w - eta * acc; acc = np.zeros_like(w); cnt = 0; updates += 1
    assert np.allclose(st.w, w, rtol=0, atol=1e-15)
    assert max(stal) == 1 and min(stal) == 0               # staleness is counted in updates


def test_sequence_pool_equals_the_stacked_microbatch():
    """The full-size GPU parity tests evaluate the oracle one sequence per process (seqpool.py):
    a stale schedule through that harness must give what oracle.stage.Stage gives on the whole
    microbatch (sequences are independent; the parameter gradient is their sum)."""
    from seqpool import PooledStage, SeqPool
    L, d, h, f, S, mb, tau, eta = 2, 16, 2, 24, 6, 3, 2, 0.05
    rng = np.random.default_rng(3)
    P = blocks.num_params(blocks.decoder_param_shapes(L, d, f))
    w0 = rng.normal(size=P) * 0.3
    xs = [rng.normal(size=(mb, S, d)) for _ in range(5)]
    dys = [rng.normal(size=(mb, S, d)) for _ in range(5)]
    with SeqPool(L, d, h, f, S, mb, workers=2) as pool:        # 2 workers, 3 sequences: one worker sums two
        a = stage.Stage("decoder", tau, eta, w0, n_blocks=L, d=d, h=h, f=f)
        b = PooledStage(pool, "decoder", tau, eta, w0, n_blocks=L, d=d, h=h, f=f)
        for t in range(5 + tau):
            if t < 5:
                assert np.allclose(a.forward(t, xs[t]), b.forward(t, xs[t]), rtol=0, atol=1e-13)
            j = t - tau
            if j >= 0:
                assert np.allclose(a.backward(j, dys[j]), b.backward(j, dys[j]), rtol=0, atol=1e-13)
                assert np.allclose(a.last_grad, b.last_grad, rtol=1e-12, atol=1e-13)
                assert a.last_staleness == b.last_staleness == min(j, tau)
        assert np.allclose(a.w, b.w, rtol=0, atol=1e-13)
