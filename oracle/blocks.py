"""Block functions of a stage and their exact reverse-mode derivatives (fp64).

TEST INFRASTRUCTURE ONLY - see oracle/__init__.py.

What a peer's forward_pass and its gradient are (paper Alg. 1; Eq. 2 defines
the gradient as the true gradient of the loss with respect to the peer's
block, evaluated at the parameters its forward used).  The paper leaves the
layer types to the model; the two used here are

* MLP stage: Linear -> ReLU -> ... -> Linear (no activation after the last).
* pre-LN transformer decoder block (L of them per stage):
      u  = LN1(x);  qkv = u Wqkv + bqkv;  a = CausalSoftmax(q k^T / sqrt(dh)) v
      x1 = x + a Wo + bo
      v2 = LN2(x1); z = v2 W1 + b1; g = GELU(z);  y = x1 + g W2 + b2
  LayerNorm uses the biased variance and eps inside the square root; GELU is
  the exact erf form; the mask keeps key j <= query i.

Everything is written as the textbook definition: numpy matmul / einsum are
the only library steps, there is no blocking or fusion.

Canonical flat parameter order (shared contract with the library, stated in
include/rv.h): layers in forward order;
  MLP:     W[in,out] row-major, b[out] per Linear.
  decoder: ln1.g, ln1.b, Wqkv[d,3d], bqkv[3d], Wo[d,d], bo[d], ln2.g, ln2.b,
           W1[d,f], b1[f], W2[f,d], b2[d] per block.
"""
import numpy as np
from scipy.special import erf

F64 = np.float64


# ----------------------------------------------------------------------------
# parameter views
# ----------------------------------------------------------------------------
def mlp_param_shapes(dims):
    shapes = []
    for i in range(len(dims) - 1):
        shapes.append((f"W{i}", (dims[i], dims[i + 1])))
        shapes.append((f"b{i}", (dims[i + 1],)))
    return shapes


def decoder_block_shapes(d, f):
    return [("ln1_g", (d,)), ("ln1_b", (d,)), ("Wqkv", (d, 3 * d)), ("bqkv", (3 * d,)),
            ("Wo", (d, d)), ("bo", (d,)), ("ln2_g", (d,)), ("ln2_b", (d,)),
            ("W1", (d, f)), ("b1", (f,)), ("W2", (f, d)), ("b2", (d,))]


def decoder_param_shapes(n_blocks, d, f):
    out = []
    for l in range(n_blocks):
        out += [(f"blk{l}.{n}", s) for n, s in decoder_block_shapes(d, f)]
    return out


def num_params(shapes):
    return int(sum(int(np.prod(s)) for _, s in shapes))


def unflatten(flat, shapes):
    """Views (no copies) of a flat vector in canonical order."""
    out, off = {}, 0
    for name, s in shapes:
        n = int(np.prod(s))
        out[name] = flat[off:off + n].reshape(s)
        off += n
    assert off == flat.size
    return out


# ----------------------------------------------------------------------------
# elementary pieces
# ----------------------------------------------------------------------------
def layernorm_fwd(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    r = 1.0 / np.sqrt(var + eps)
    xh = (x - mu) * r
    return xh * g + b, (xh, r)


def layernorm_bwd(dy, g, cache):
    xh, r = cache
    dxh = dy * g
    dg = (dy * xh).reshape(-1, xh.shape[-1]).sum(axis=0)
    db = dy.reshape(-1, xh.shape[-1]).sum(axis=0)
    dx = r * (dxh - dxh.mean(axis=-1, keepdims=True)
              - xh * (dxh * xh).mean(axis=-1, keepdims=True))
    return dx, dg, db


def gelu(z):
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def gelu_grad(z):
    # d/dz [ z Phi(z) ] = Phi(z) + z phi(z)
    return 0.5 * (1.0 + erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def causal_attention_fwd(q, k, v):
    """q,k,v: [mb,h,S,dh].  Returns a [mb,h,S,dh] and the probabilities."""
    S, dh = q.shape[-2], q.shape[-1]
    s = (q @ np.swapaxes(k, -1, -2)) / np.sqrt(float(dh))          # s[i,j] = q_i . k_j / sqrt(dh)
    i = np.arange(S)[:, None]
    j = np.arange(S)[None, :]
    s = np.where(j <= i, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    p = e / e.sum(axis=-1, keepdims=True)
    return p @ v, p                                               # a_i = sum_j p_ij v_j


def causal_attention_bwd(da, q, k, v, p):
    dh = q.shape[-1]
    pt = np.swapaxes(p, -1, -2)
    dv = pt @ da                                                  # dv_j = sum_i p_ij da_i
    dp = da @ np.swapaxes(v, -1, -2)                              # dp_ij = da_i . v_j
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dq = (ds @ k) / np.sqrt(float(dh))                            # dq_i = sum_j ds_ij k_j / sqrt(dh)
    dk = (np.swapaxes(ds, -1, -2) @ q) / np.sqrt(float(dh))       # dk_j = sum_i ds_ij q_i / sqrt(dh)
    return dq, dk, dv


def _split_heads(t, h):
    mb, S, d = t.shape
    return t.reshape(mb, S, h, d // h).transpose(0, 2, 1, 3)


def _merge_heads(t):
    mb, h, S, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(mb, S, h * dh)


# ----------------------------------------------------------------------------
# MLP stage
# ----------------------------------------------------------------------------
def mlp_forward(flat_w, dims, x):
    """x: [rows, dims[0]] -> [rows, dims[-1]]; ReLU between Linears."""
    p = unflatten(flat_w, mlp_param_shapes(dims))
    a = x
    n = len(dims) - 1
    for i in range(n):
        a = a @ p[f"W{i}"] + p[f"b{i}"]
        if i < n - 1:
            a = np.maximum(a, 0.0)
    return a


def mlp_backward(flat_w, dims, x, dy):
    """Returns (dx, flat gradient in canonical order)."""
    shapes = mlp_param_shapes(dims)
    p = unflatten(flat_w, shapes)
    n = len(dims) - 1
    acts, pre = [x], []
    a = x
    for i in range(n):
        zlin = a @ p[f"W{i}"] + p[f"b{i}"]
        pre.append(zlin)
        a = np.maximum(zlin, 0.0) if i < n - 1 else zlin
        acts.append(a)
    g = np.zeros(flat_w.size, dtype=F64)
    gp = unflatten(g, shapes)
    d = dy
    for i in reversed(range(n)):
        if i < n - 1:
            d = d * (pre[i] > 0.0)
        gp[f"W{i}"][...] = acts[i].T @ d
        gp[f"b{i}"][...] = d.sum(axis=0)
        d = d @ p[f"W{i}"].T
    return d, g


# ----------------------------------------------------------------------------
# decoder stage
# ----------------------------------------------------------------------------
def decoder_block_forward(p, x, h, eps, keep=False):
    u, c1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = u @ p["Wqkv"] + p["bqkv"]
    d = x.shape[-1]
    q, k, v = (_split_heads(qkv[..., i * d:(i + 1) * d], h) for i in range(3))
    a4, prob = causal_attention_fwd(q, k, v)
    a = _merge_heads(a4)
    x1 = x + a @ p["Wo"] + p["bo"]
    v2, c2 = layernorm_fwd(x1, p["ln2_g"], p["ln2_b"], eps)
    z = v2 @ p["W1"] + p["b1"]
    g = gelu(z)
    y = x1 + g @ p["W2"] + p["b2"]
    if keep:
        return y, dict(c1=c1, u=u, q=q, k=k, v=v, prob=prob, a=a, c2=c2, v2=v2, z=z, g=g)
    return y


def decoder_block_backward(p, gp, cache, dy, h):
    """Fills gp (views into the flat gradient) and returns dx."""
    d = dy.shape[-1]
    T = dy.shape[0] * dy.shape[1]
    f2 = lambda t: t.reshape(T, -1)
    gp["W2"][...] = f2(cache["g"]).T @ f2(dy)
    gp["b2"][...] = f2(dy).sum(axis=0)
    dg = dy @ p["W2"].T
    dz = dg * gelu_grad(cache["z"])
    gp["W1"][...] = f2(cache["v2"]).T @ f2(dz)
    gp["b1"][...] = f2(dz).sum(axis=0)
    dv2 = dz @ p["W1"].T
    dln, dgam, dbet = layernorm_bwd(dv2, p["ln2_g"], cache["c2"])
    gp["ln2_g"][...] = dgam
    gp["ln2_b"][...] = dbet
    dx1 = dy + dln
    gp["Wo"][...] = f2(cache["a"]).T @ f2(dx1)
    gp["bo"][...] = f2(dx1).sum(axis=0)
    da = _split_heads(dx1 @ p["Wo"].T, h)
    dq, dk, dv = causal_attention_bwd(da, cache["q"], cache["k"], cache["v"], cache["prob"])
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1)
    gp["Wqkv"][...] = f2(cache["u"]).T @ f2(dqkv)
    gp["bqkv"][...] = f2(dqkv).sum(axis=0)
    du = dqkv @ p["Wqkv"].T
    dln, dgam, dbet = layernorm_bwd(du, p["ln1_g"], cache["c1"])
    gp["ln1_g"][...] = dgam
    gp["ln1_b"][...] = dbet
    return dx1 + dln


def decoder_forward(flat_w, n_blocks, d, h, f, eps, x):
    """x: [mb,S,d] -> [mb,S,d]."""
    p = unflatten(flat_w, decoder_param_shapes(n_blocks, d, f))
    for l in range(n_blocks):
        pl = {n: p[f"blk{l}.{n}"] for n, _ in decoder_block_shapes(d, f)}
        x = decoder_block_forward(pl, x, h, eps)
    return x


def decoder_backward(flat_w, n_blocks, d, h, f, eps, x, dy):
    """Recomputes the forward from (flat_w, x), then returns (dx, flat grad)."""
    shapes = decoder_param_shapes(n_blocks, d, f)
    p = unflatten(flat_w, shapes)
    g = np.zeros(flat_w.size, dtype=F64)
    gp = unflatten(g, shapes)
    names = [n for n, _ in decoder_block_shapes(d, f)]
    caches = []
    for l in range(n_blocks):
        pl = {n: p[f"blk{l}.{n}"] for n in names}
        x, c = decoder_block_forward(pl, x, h, eps, keep=True)
        caches.append(c)
    for l in reversed(range(n_blocks)):
        pl = {n: p[f"blk{l}.{n}"] for n in names}
        gl = {n: gp[f"blk{l}.{n}"] for n in names}
        dy = decoder_block_backward(pl, gl, caches.pop(), dy, h)
    return dy, g
