"""Pins for oracle/layer.py: finite differences, torch autograd on an independently
written forward, brute force on tiny inputs, closed-form special cases."""
import math

import numpy as np
import pytest
import torch

from oracle import layer as L

RNG = np.random.default_rng(7)


def _params(h, f, scale=0.3):
    p = {}
    for k, shp in L.param_shapes(h, f).items():
        a = RNG.standard_normal(shp) * scale
        if k.endswith("_g"):
            a = 1.0 + a
        p[k] = a
    return p


# ------------------------------------------------------------------ whole layer
def _loss(p, x, dy, a, causal):
    y, _ = L.layer_fwd(p, x, a, 1e-5, causal)
    return float((y * dy).sum())


@pytest.mark.parametrize("causal", [True, False])
def test_layer_backward_finite_differences(causal):
    h, a, f, S_seq, S_mb = 16, 2, 64, 8, 2
    p = _params(h, f)
    x = RNG.standard_normal((S_mb, S_seq, h))
    dy = RNG.standard_normal((S_mb, S_seq, h))
    y, cache = L.layer_fwd(p, x, a, 1e-5, causal)
    dx, G = L.layer_bwd(p, cache, dy, a)
    eps = 1e-5
    for name, analytic in list(G.items()) + [("x", dx)]:
        target = x if name == "x" else p[name]
        flat = target.reshape(-1)
        idx = RNG.choice(flat.size, size=min(24, flat.size), replace=False)
        for i in idx:
            old = flat[i]
            flat[i] = old + eps
            lp = _loss(p, x, dy, a, causal)
            flat[i] = old - eps
            lm = _loss(p, x, dy, a, causal)
            flat[i] = old
            fd = (lp - lm) / (2 * eps)
            an = analytic.reshape(-1)[i]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, i, fd, an)


def _torch_layer(p, x, a, causal, eps):
    """The same block written with torch library ops (autograd gives the gradients)."""
    F = torch.nn.functional
    h = x.shape[-1]
    t = F.layer_norm(x, (h,), p["ln1_g"], p["ln1_b"], eps)
    qkv = t @ p["w_qkv"] + p["b_qkv"]
    q, k, v = qkv.split(h, dim=-1)
    B, S, _ = x.shape
    sh = lambda z: z.view(B, S, a, h // a).transpose(1, 2)
    o = F.scaled_dot_product_attention(sh(q), sh(k), sh(v), is_causal=causal)
    o = o.transpose(1, 2).reshape(B, S, h)
    x1 = x + o @ p["w_o"] + p["b_o"]
    c = F.layer_norm(x1, (h,), p["ln2_g"], p["ln2_b"], eps)
    u = c @ p["w_fc1"] + p["b_fc1"]
    return x1 + F.gelu(u, approximate="tanh") @ p["w_fc2"] + p["b_fc2"]


@pytest.mark.parametrize("causal", [True, False])
def test_layer_against_torch_autograd(causal):
    h, a, f, S_seq, S_mb = 32, 4, 128, 12, 3
    p = _params(h, f)
    x = RNG.standard_normal((S_mb, S_seq, h))
    dy = RNG.standard_normal((S_mb, S_seq, h))
    y, cache = L.layer_fwd(p, x, a, 1e-5, causal)
    dx, G = L.layer_bwd(p, cache, dy, a)
    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = _torch_layer(tp, tx, a, causal, 1e-5)
    (ty * torch.tensor(dy)).sum().backward()
    assert np.allclose(y, ty.detach().numpy(), rtol=1e-10, atol=1e-10)
    assert np.allclose(dx, tx.grad.numpy(), rtol=1e-9, atol=1e-10)
    for k in G:
        assert np.allclose(G[k], tp[k].grad.numpy(), rtol=1e-9, atol=1e-10), k


def test_identity_linears_and_packing():
    # With LN gains 1/biases 0 and w_o = 0, w_fc2 = 0 the layer is the identity plus biases
    h, a, f = 8, 2, 32
    p = _params(h, f)
    p["w_o"][:] = 0
    p["w_fc2"][:] = 0
    x = RNG.standard_normal((1, 5, h))
    y, _ = L.layer_fwd(p, x, a)
    assert np.allclose(y, x + p["b_o"] + p["b_fc2"])
    # Q|K|V packing and head ownership: ctx of head j depends only on columns j*d..(j+1)*d of each third
    qkv = RNG.standard_normal((1, 5, 3 * h))
    ctx, _ = L.attention_fwd(qkv, a, True)
    qkv2 = qkv.copy()
    d = h // a
    qkv2[..., 0:d] += 1.0            # perturb Q of head 0 only
    ctx2, _ = L.attention_fwd(qkv2, a, True)
    assert not np.allclose(ctx[..., :d], ctx2[..., :d])
    assert np.array_equal(ctx[..., d:], ctx2[..., d:])


# -------------------------------------------------------------------- attention
def test_attention_brute_force_noncausal_single_head():
    S, d = 6, 4
    qkv = RNG.standard_normal((1, S, 3 * d))
    ctx, _ = L.attention_fwd(qkv, 1, causal=False)
    q, k, v = qkv[0, :, :d], qkv[0, :, d:2 * d], qkv[0, :, 2 * d:]
    for i in range(S):
        w = [math.exp(sum(q[i, c] * k[j, c] for c in range(d)) / math.sqrt(d)) for j in range(S)]
        z = sum(w)
        for c in range(d):
            ref = sum(w[j] * v[j, c] for j in range(S)) / z
            assert abs(ctx[0, i, c] - ref) < 1e-12


def test_attention_causal_special_cases():
    S, h, a = 7, 8, 2
    qkv = RNG.standard_normal((2, S, 3 * h))
    ctx, _ = L.attention_fwd(qkv, a, causal=True)
    # position 0 sees only itself
    assert np.allclose(ctx[:, 0], qkv[:, 0, 2 * h:])
    # Q = K = 0: uniform weights over the prefix -> running mean of V
    qkv0 = qkv.copy()
    qkv0[..., :2 * h] = 0
    ctx0, _ = L.attention_fwd(qkv0, a, causal=True)
    run = np.cumsum(qkv0[..., 2 * h:], axis=1) / np.arange(1, S + 1)[None, :, None]
    assert np.allclose(ctx0, run)
    # causal: output at i does not change when later positions change
    qkv1 = qkv.copy()
    qkv1[:, 4:] += 3.0
    ctx1, _ = L.attention_fwd(qkv1, a, causal=True)
    assert np.array_equal(ctx[:, :4], ctx1[:, :4])


# -------------------------------------------------------------------- LayerNorm
def test_layernorm_moments_and_gradient_identities():
    n = 24
    x = RNG.standard_normal((5, n)) * 3 + 1
    eps = 1e-5
    y, saved = L.layernorm_fwd(x, np.ones(n), np.zeros(n), eps)
    var = x.var(axis=-1)
    assert np.allclose(y.mean(axis=-1), 0, atol=1e-12)
    assert np.allclose(y.var(axis=-1), var / (var + eps))
    # sum_i y_i is constant in x (gain 1): gradient of it w.r.t. x is zero
    dx, dg, db = L.layernorm_bwd(np.ones_like(x), np.ones(n), saved)
    assert np.allclose(dx, 0, atol=1e-12)
    # gain/bias gradients are plain column sums
    g = RNG.standard_normal(n)
    dy = RNG.standard_normal(x.shape)
    y2, saved2 = L.layernorm_fwd(x, g, np.zeros(n), eps)
    _, dg, db = L.layernorm_bwd(dy, g, saved2)
    xhat = (x - x.mean(-1, keepdims=True)) / np.sqrt(var + eps)[:, None]
    for j in range(n):
        assert abs(dg[j] - sum(dy[i, j] * xhat[i, j] for i in range(5))) < 1e-12
        assert abs(db[j] - sum(dy[i, j] for i in range(5))) < 1e-12


# ------------------------------------------------------------------------- GeLU
def test_gelu_values_and_forms():
    assert L.gelu(np.array(0.0)) == 0.0
    assert L.gelu_grad(np.array(0.0)) == 0.5
    big = np.array([8.0, -8.0])
    assert np.allclose(L.gelu(big), [8.0, 0.0], atol=1e-9)
    u = np.linspace(-6, 6, 2001)
    assert np.max(np.abs(L.gelu(u, "tanh") - L.gelu(u, "erf"))) < 1e-3
    t = torch.tensor(u, dtype=torch.float64, requires_grad=True)
    g = torch.nn.functional.gelu(t, approximate="tanh")
    g.sum().backward()
    assert np.allclose(L.gelu(u), g.detach().numpy(), atol=1e-14)
    assert np.allclose(L.gelu_grad(u), t.grad.numpy(), atol=1e-13)
    # erf form derivative by central differences
    e = 1e-6
    fd = (L.gelu(u + e, "erf") - L.gelu(u - e, "erf")) / (2 * e)
    assert np.allclose(L.gelu_grad(u, "erf"), fd, atol=1e-8)
