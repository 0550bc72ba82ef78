"""One transformer layer, forward and backward, in float64 numpy.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper (App. A.1, "Setup") fixes only the outline: identical transformer
layers of hidden size S_hidden, multi-head self-attention with N_heads heads of
size S_head (N_heads * S_head = S_hidden) followed by a two-layer MLP of hidden
size S_mlp.  The finer readings taken here:

  * pre-LN GPT block:  x1 = x  + Attn(LN1(x)) W_o + b_o
                       y  = x1 + GeLU(LN2(x1) W_fc1 + b_fc1) W_fc2 + b_fc2
  * biases on all four linears, LayerNorm with gain and bias, eps inside sqrt
  * W_qkv columns are [Q | K | V]; head a owns columns a*S_head..(a+1)*S_head-1
    of each third
  * softmax scale 1/sqrt(S_head); causal mask excludes j > i (not "-inf added")
  * GeLU in its tanh form (the erf form is available through `gelu="erf"`)
  * no dropout

Everything is written as the plain definition: full S_seq x S_seq probability
matrices are formed, nothing is tiled or fused.
"""
import math

import numpy as np

PARAM_NAMES = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2",
)


def param_shapes(S_hidden, S_mlp):
    h, f = S_hidden, S_mlp
    return {
        "ln1_g": (h,), "ln1_b": (h,),
        "w_qkv": (h, 3 * h), "b_qkv": (3 * h,),
        "w_o": (h, h), "b_o": (h,),
        "ln2_g": (h,), "ln2_b": (h,),
        "w_fc1": (h, f), "b_fc1": (f,),
        "w_fc2": (f, h), "b_fc2": (h,),
    }


# --------------------------------------------------------------------------- GeLU
_K0 = math.sqrt(2.0 / math.pi)
_K1 = 0.044715


def gelu(u, form="tanh"):
    if form == "tanh":
        return 0.5 * u * (1.0 + np.tanh(_K0 * (u + _K1 * u ** 3)))
    if form == "erf":
        from scipy.special import erf
        return 0.5 * u * (1.0 + erf(u / math.sqrt(2.0)))
    raise ValueError(form)


def gelu_grad(u, form="tanh"):
    """d gelu(u) / du."""
    if form == "tanh":
        t = np.tanh(_K0 * (u + _K1 * u ** 3))
        dt = (1.0 - t * t) * _K0 * (1.0 + 3.0 * _K1 * u * u)
        return 0.5 * (1.0 + t) + 0.5 * u * dt
    if form == "erf":
        from scipy.special import erf
        return 0.5 * (1.0 + erf(u / math.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
    raise ValueError(form)


# ---------------------------------------------------------------------- LayerNorm
def layernorm_fwd(x, g, b, eps):
    """y = (x - mean) / sqrt(var + eps) * g + b over the last axis (biased var)."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * g + b, (xhat, rstd)


def layernorm_bwd(dy, g, saved):
    """Returns dx, dg, db given the upstream dy."""
    xhat, rstd = saved
    n = dy.shape[-1]
    dxhat = dy * g
    dg = (dy * xhat).reshape(-1, n).sum(axis=0)
    db = dy.reshape(-1, n).sum(axis=0)
    # d/dx of (x - mu) * rstd, applied to dxhat
    s1 = dxhat.sum(axis=-1, keepdims=True)
    s2 = (dxhat * xhat).sum(axis=-1, keepdims=True)
    dx = rstd * (dxhat - s1 / n - xhat * s2 / n)
    return dx, dg, db


# ---------------------------------------------------------------------- attention
def _split_heads(t, N_heads):
    # [S_mb, S_seq, S_hidden] -> [S_mb, N_heads, S_seq, S_head]
    S_mb, S_seq, h = t.shape
    return t.reshape(S_mb, S_seq, N_heads, h // N_heads).transpose(0, 2, 1, 3)


def _merge_heads(t):
    S_mb, a, S_seq, d = t.shape
    return t.transpose(0, 2, 1, 3).reshape(S_mb, S_seq, a * d)


def attention_fwd(qkv, N_heads, causal=True):
    """softmax(Q K^T / sqrt(S_head) [+ causal mask]) V per head.

    qkv: [S_mb, S_seq, 3*S_hidden] packed [Q | K | V].
    Returns ctx [S_mb, S_seq, S_hidden] and what the backward needs.
    """
    h = qkv.shape[-1] // 3
    S_seq = qkv.shape[1]
    q = _split_heads(qkv[..., 0 * h:1 * h], N_heads)
    k = _split_heads(qkv[..., 1 * h:2 * h], N_heads)
    v = _split_heads(qkv[..., 2 * h:3 * h], N_heads)
    d = q.shape[-1]
    s = np.matmul(q, k.transpose(0, 1, 3, 2)) / math.sqrt(d)
    if causal:
        allowed = np.tril(np.ones((S_seq, S_seq), dtype=bool))
        s = np.where(allowed, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)                       # exp(-inf) = 0: masked entries drop out
    p = e / e.sum(axis=-1, keepdims=True)
    ctx = _merge_heads(np.matmul(p, v))
    return ctx, (q, k, v, p)


def attention_bwd(dctx, saved, N_heads):
    """Returns dqkv [S_mb, S_seq, 3*S_hidden]."""
    q, k, v, p = saved
    d = q.shape[-1]
    do = _split_heads(dctx, N_heads)
    dv = np.matmul(p.transpose(0, 1, 3, 2), do)
    dp = np.matmul(do, v.transpose(0, 1, 3, 2))
    # softmax Jacobian: ds = p * (dp - sum_j p_j dp_j); masked p are 0 so ds is 0 there
    ds = p * (dp - (p * dp).sum(axis=-1, keepdims=True))
    ds = ds / math.sqrt(d)
    dq = np.matmul(ds, k)
    dk = np.matmul(ds.transpose(0, 1, 3, 2), q)
    return np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1)


# -------------------------------------------------------------------------- layer
def layer_fwd(p, x, N_heads, eps=1e-5, causal=True, gelu_form="tanh"):
    """x: [S_mb, S_seq, S_hidden] -> y (same shape), cache for the backward."""
    a, ln1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = a @ p["w_qkv"] + p["b_qkv"]
    ctx, att = attention_fwd(qkv, N_heads, causal)
    x1 = x + ctx @ p["w_o"] + p["b_o"]
    c, ln2 = layernorm_fwd(x1, p["ln2_g"], p["ln2_b"], eps)
    u = c @ p["w_fc1"] + p["b_fc1"]
    g = gelu(u, gelu_form)
    y = x1 + g @ p["w_fc2"] + p["b_fc2"]
    cache = dict(a=a, ln1=ln1, att=att, ctx=ctx, c=c, ln2=ln2, u=u, g=g, gelu_form=gelu_form)
    return y, cache


def _flat(t):
    return t.reshape(-1, t.shape[-1])


def layer_bwd(p, cache, dy, N_heads):
    """Returns dx and a dict of parameter gradients for this one micro-batch."""
    G = {}
    # y = x1 + g W_fc2 + b_fc2
    G["w_fc2"] = _flat(cache["g"]).T @ _flat(dy)
    G["b_fc2"] = _flat(dy).sum(axis=0)
    dg = dy @ p["w_fc2"].T
    du = dg * gelu_grad(cache["u"], cache["gelu_form"])
    G["w_fc1"] = _flat(cache["c"]).T @ _flat(du)
    G["b_fc1"] = _flat(du).sum(axis=0)
    dc = du @ p["w_fc1"].T
    dx1_ln, G["ln2_g"], G["ln2_b"] = layernorm_bwd(dc, p["ln2_g"], cache["ln2"])
    dx1 = dy + dx1_ln
    # x1 = x + ctx W_o + b_o
    G["w_o"] = _flat(cache["ctx"]).T @ _flat(dx1)
    G["b_o"] = _flat(dx1).sum(axis=0)
    dctx = dx1 @ p["w_o"].T
    dqkv = attention_bwd(dctx, cache["att"], N_heads)
    G["w_qkv"] = _flat(cache["a"]).T @ _flat(dqkv)
    G["b_qkv"] = _flat(dqkv).sum(axis=0)
    da = dqkv @ p["w_qkv"].T
    dx_ln, G["ln1_g"], G["ln1_b"] = layernorm_bwd(da, p["ln1_g"], cache["ln1"])
    dx = dx1 + dx_ln
    return dx, G
