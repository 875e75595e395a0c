"""Pins for oracle/blocks.py: finite differences, invariants, textbook cases."""
import numpy as np
import pytest

from oracle import blocks

EPS = 1e-5


def _fd_check(loss, w, g, h=1e-6, tol=2e-7):
    """Central differences on every coordinate; error relative to the gradient's scale."""
    scale = np.abs(g).max()
    worst = 0.0
    for i in range(w.size):
        wp = w.copy(); wp.flat[i] += h
        wm = w.copy(); wm.flat[i] -= h
        fd = (loss(wp) - loss(wm)) / (2 * h)
        worst = max(worst, abs(fd - g.flat[i]) / scale)
    assert worst < tol, worst


def test_mlp_gradients_finite_differences():
    rng = np.random.default_rng(1)
    dims = [4, 6, 5, 3]
    P = blocks.num_params(blocks.mlp_param_shapes(dims))
    w = rng.normal(size=P) * 0.5
    x = rng.normal(size=(5, 4))
    dy = rng.normal(size=(5, 3))
    dx, g = blocks.mlp_backward(w, dims, x, dy)
    _fd_check(lambda w_: (blocks.mlp_forward(w_, dims, x) * dy).sum(), w, g)
    _fd_check(lambda x_: (blocks.mlp_forward(w, dims, x_) * dy).sum(), x, dx)


def test_decoder_gradients_finite_differences():
    rng = np.random.default_rng(2)
    L, d, h, f, S, mb = 2, 8, 2, 16, 4, 2
    P = blocks.num_params(blocks.decoder_param_shapes(L, d, f))
    assert P == L * (4 * d * d + 2 * d * f + 9 * d + f)
    w = rng.normal(size=P) * 0.3
    x = rng.normal(size=(mb, S, d))
    dy = rng.normal(size=(mb, S, d))
    dx, g = blocks.decoder_backward(w, L, d, h, f, EPS, x, dy)
    _fd_check(lambda w_: (blocks.decoder_forward(w_, L, d, h, f, EPS, x) * dy).sum(), w, g, tol=5e-7)
    _fd_check(lambda x_: (blocks.decoder_forward(w, L, d, h, f, EPS, x_) * dy).sum(), x, dx, tol=5e-7)


def test_decoder_matches_torch_autograd():
    """Independent cross-check of the whole block against an fp64 autograd graph."""
    import torch
    rng = np.random.default_rng(3)
    L, d, h, f, S, mb = 2, 12, 3, 20, 5, 2
    shapes = blocks.decoder_param_shapes(L, d, f)
    w = rng.normal(size=blocks.num_params(shapes)) * 0.3
    x = rng.normal(size=(mb, S, d)); dy = rng.normal(size=(mb, S, d))
    wt = torch.tensor(w, requires_grad=True); xt = torch.tensor(x, requires_grad=True)
    off = 0; p = {}
    for n, s in shapes:
        k = int(np.prod(s)); p[n] = wt[off:off + k].reshape(s); off += k
    a = xt
    for l in range(L):
        g = lambda n: p[f"blk{l}.{n}"]
        u = torch.nn.functional.layer_norm(a, (d,), g("ln1_g"), g("ln1_b"), EPS)
        qkv = u @ g("Wqkv") + g("bqkv")
        q, k, v = [t.reshape(mb, S, h, d // h).transpose(1, 2) for t in qkv.split(d, dim=-1)]
        at = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
        a = a + at.transpose(1, 2).reshape(mb, S, d) @ g("Wo") + g("bo")
        v2 = torch.nn.functional.layer_norm(a, (d,), g("ln2_g"), g("ln2_b"), EPS)
        a = a + torch.nn.functional.gelu(v2 @ g("W1") + g("b1")) @ g("W2") + g("b2")
    (a * torch.tensor(dy)).sum().backward()
    y = blocks.decoder_forward(w, L, d, h, f, EPS, x)
    dx, gr = blocks.decoder_backward(w, L, d, h, f, EPS, x, dy)
    assert np.allclose(y, a.detach().numpy(), rtol=1e-11, atol=1e-12)
    assert np.allclose(dx, xt.grad.numpy(), rtol=1e-10, atol=1e-12)
    assert np.allclose(gr, wt.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_causal_mask_invariance():
    rng = np.random.default_rng(4)
    L, d, h, f, S, mb = 1, 8, 2, 16, 6, 2
    w = rng.normal(size=blocks.num_params(blocks.decoder_param_shapes(L, d, f))) * 0.3
    x = rng.normal(size=(mb, S, d))
    y = blocks.decoder_forward(w, L, d, h, f, EPS, x)
    x2 = x.copy(); x2[:, 4:, :] += rng.normal(size=(mb, 2, d))   # change the future of i <= 3
    y2 = blocks.decoder_forward(w, L, d, h, f, EPS, x2)
    assert np.array_equal(y[:, :4], y2[:, :4]) and not np.allclose(y[:, 4:], y2[:, 4:])
    dy = rng.normal(size=(mb, S, d))
    dx, _ = blocks.decoder_backward(w, L, d, h, f, EPS, x, dy)
    dy2 = dy.copy(); dy2[:, :3, :] += 1.0                       # change grads of the past of j >= 3
    dx2, _ = blocks.decoder_backward(w, L, d, h, f, EPS, x, dy2)
    assert np.array_equal(dx[:, 3:], dx2[:, 3:])


def test_softmax_rows_and_single_token_attention():
    rng = np.random.default_rng(5)
    q, k, v = (rng.normal(size=(2, 3, 7, 4)) for _ in range(3))
    a, p = blocks.causal_attention_fwd(q, k, v)
    assert np.allclose(p.sum(-1), 1.0, atol=1e-14)
    assert np.all(np.triu(p[0, 0], 1) == 0.0)
    assert np.allclose(a[:, :, 0], v[:, :, 0])                  # first query sees only key 0
    # uniform scores -> running mean of v over the visible prefix
    a2, _ = blocks.causal_attention_fwd(np.zeros_like(q), k, v)
    assert np.allclose(a2[0, 0, 4], v[0, 0, :5].mean(axis=0))
    # S = 1: attention is the identity on v
    a1, _ = blocks.causal_attention_fwd(q[:, :, :1], k[:, :, :1], v[:, :, :1])
    assert np.array_equal(a1, v[:, :, :1])
    # the 1/sqrt(dh) scale: two keys, dh = 4, q.k = 2 vs 0 -> p = sigmoid(2/2)
    qq = np.zeros((1, 1, 2, 4)); kk = np.zeros((1, 1, 2, 4)); qq[0, 0, 1, 0] = 2.0; kk[0, 0, 1, 0] = 1.0
    _, pp = blocks.causal_attention_fwd(qq, kk, kk)
    assert np.isclose(pp[0, 0, 1, 1], 1.0 / (1.0 + np.exp(-1.0)))


def test_layernorm_statistics():
    rng = np.random.default_rng(6)
    x = rng.normal(size=(3, 5, 16)) * 2.0 + 1.0
    eps = 1e-2
    y, (xh, r) = blocks.layernorm_fwd(x, np.ones(16), np.zeros(16), eps)
    var = x.var(axis=-1)
    assert np.allclose(y.mean(-1), 0.0, atol=1e-14)
    assert np.allclose(y.var(-1), var / (var + eps))
    g = rng.normal(size=16); b = rng.normal(size=16)
    y2, _ = blocks.layernorm_fwd(x, g, b, eps)
    assert np.allclose(y2, y * g + b)


def test_gelu_values():
    # closed forms: GELU(0)=0, GELU'(0)=1/2, GELU(z)-GELU(-z)=z, tails
    assert blocks.gelu(np.array(0.0)) == 0.0
    assert blocks.gelu_grad(np.array(0.0)) == 0.5
    z = np.linspace(-4, 4, 33)
    assert np.allclose(blocks.gelu(z) - blocks.gelu(-z), z)
    assert np.isclose(blocks.gelu(np.array(1.0)), 0.8413447460685429)    # Phi(1)
    assert np.isclose(blocks.gelu(np.array(10.0)), 10.0) and abs(blocks.gelu(np.array(-10.0))) < 1e-20
    h = 1e-6
    assert np.allclose((blocks.gelu(z + h) - blocks.gelu(z - h)) / (2 * h), blocks.gelu_grad(z), atol=1e-9)


def test_single_linear_textbook_case():
    rng = np.random.default_rng(7)
    dims = [5, 3]
    W = rng.normal(size=(5, 3)); b = rng.normal(size=3)
    w = np.concatenate([W.ravel(), b])
    x = rng.normal(size=(4, 5)); dy = rng.normal(size=(4, 3))
    assert np.allclose(blocks.mlp_forward(w, dims, x), x @ W + b)
    dx, g = blocks.mlp_backward(w, dims, x, dy)
    assert np.allclose(dx, dy @ W.T)
    assert np.allclose(g[:15].reshape(5, 3), x.T @ dy) and np.allclose(g[15:], dy.sum(0))


def test_relu_gate_and_param_count_of_paper_sized_mlp():
    dims = [64, 128, 64]
    assert blocks.num_params(blocks.mlp_param_shapes(dims)) == 16576
    # a negative pre-activation passes no gradient
    w = np.array([1.0, 0.0, 1.0, 0.0])          # 1 -> 1 -> 1 : W0=1,b0=0,W1=1,b1=0
    dx, g = blocks.mlp_backward(w, [1, 1, 1], np.array([[-2.0]]), np.array([[1.0]]))
    assert dx[0, 0] == 0.0 and g[0] == 0.0 and g[2] == 0.0 and g[3] == 1.0
