"""Transformer layer forward / backward in float64 (oracle; test infrastructure).

The paper (Section 5.1) defines FRC/BRC on node n as exactly the computation
FNC/BNC of node n+1 over the same parameters; it does not spell out the layer
math, which is the textbook transformer layer of the models it trains
(Section 7, Table 1: BERT-Large, GPT-2).  This file writes that definition out
step by step.  Every function is the plain formula; numpy's matmul is the only
library primitive.

Parameter layout of one layer (flat, in this order; matrices are [in, out]
row-major so that Y = X @ W):
  Wqkv [H,3H]  bqkv [3H]  Wo [H,H]  bo [H]  g1 [H]  be1 [H]
  W1 [H,F]  b1 [F]  W2 [F,H]  b2 [H]  g2 [H]  be2 [H]
Columns of Wqkv: [0,H) queries, [H,2H) keys, [2H,3H) values; head h owns
columns h*d .. (h+1)*d-1 of each third.

arch 0: post-LN bidirectional encoder   r1 = x + attn(x); y1 = LN1(r1);
                                        r2 = y1 + ffn(y1); y = LN2(r2)
arch 1: pre-LN causal decoder           u = LN1(x); x1 = x + attn(u);
                                        v = LN2(x1); y = x1 + ffn(v)
"""
import math

import numpy as np

try:  # erf on arrays; scipy is only a table of the special function
    from scipy.special import erf as _erf
except Exception:  # pragma: no cover
    _erf = np.vectorize(math.erf)

PARAM_NAMES = ("Wqkv", "bqkv", "Wo", "bo", "g1", "be1",
               "W1", "b1", "W2", "b2", "g2", "be2")


def param_shapes(H, F):
    return {"Wqkv": (H, 3 * H), "bqkv": (3 * H,), "Wo": (H, H), "bo": (H,),
            "g1": (H,), "be1": (H,), "W1": (H, F), "b1": (F,),
            "W2": (F, H), "b2": (H,), "g2": (H,), "be2": (H,)}


def layer_param_count(H, F):
    return 4 * H * H + 2 * H * F + 9 * H + F


def unpack_layer(flat, H, F):
    """Split one layer's flat parameter (or gradient) vector into named arrays."""
    out, off = {}, 0
    for name in PARAM_NAMES:
        shp = param_shapes(H, F)[name]
        n = int(np.prod(shp))
        out[name] = np.asarray(flat[off:off + n], dtype=np.float64).reshape(shp)
        off += n
    assert off == layer_param_count(H, F)
    return out


def pack_layer(named, H, F):
    return np.concatenate([np.asarray(named[n], dtype=np.float64).reshape(-1)
                           for n in PARAM_NAMES])


# ----------------------------------------------------------------- pieces

def layernorm_fwd(r, gamma, beta, eps):
    mu = r.mean(axis=-1, keepdims=True)
    var = ((r - mu) ** 2).mean(axis=-1, keepdims=True)        # biased variance
    rstd = 1.0 / np.sqrt(var + eps)
    rhat = (r - mu) * rstd
    return gamma * rhat + beta, (rhat, rstd)


def layernorm_bwd(dout, gamma, cache):
    rhat, rstd = cache
    dgamma = (dout * rhat).sum(axis=0)
    dbeta = dout.sum(axis=0)
    drhat = dout * gamma
    m1 = drhat.mean(axis=-1, keepdims=True)
    m2 = (drhat * rhat).mean(axis=-1, keepdims=True)
    dr = (drhat - m1 - rhat * m2) * rstd
    return dr, dgamma, dbeta


def gelu(h):
    return 0.5 * h * (1.0 + _erf(h / math.sqrt(2.0)))


def gelu_grad(h):
    return 0.5 * (1.0 + _erf(h / math.sqrt(2.0))) + h * np.exp(-0.5 * h * h) / math.sqrt(2.0 * math.pi)


def attention_fwd(qkv, B, S, n_h, causal):
    """qkv [B*S, 3H] -> ctx [B*S, H]; also returns the probabilities."""
    T, H3 = qkv.shape
    H = H3 // 3
    d = H // n_h
    ctx = np.zeros((T, H))
    probs = np.zeros((B, n_h, S, S))
    for b in range(B):
        rows = slice(b * S, (b + 1) * S)
        for h in range(n_h):
            q = qkv[rows, h * d:(h + 1) * d]
            k = qkv[rows, H + h * d:H + (h + 1) * d]
            v = qkv[rows, 2 * H + h * d:2 * H + (h + 1) * d]
            s = (q @ k.T) / math.sqrt(d)
            if causal:
                s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
            m = s.max(axis=-1, keepdims=True)
            e = np.exp(s - m)
            p = e / e.sum(axis=-1, keepdims=True)
            probs[b, h] = p
            ctx[rows, h * d:(h + 1) * d] = p @ v
    return ctx, probs


def attention_bwd(dctx, qkv, probs, B, S, n_h):
    T, H3 = qkv.shape
    H = H3 // 3
    d = H // n_h
    dqkv = np.zeros_like(qkv)
    for b in range(B):
        rows = slice(b * S, (b + 1) * S)
        for h in range(n_h):
            q = qkv[rows, h * d:(h + 1) * d]
            k = qkv[rows, H + h * d:H + (h + 1) * d]
            v = qkv[rows, 2 * H + h * d:2 * H + (h + 1) * d]
            p = probs[b, h]
            do = dctx[rows, h * d:(h + 1) * d]
            dv = p.T @ do
            dp = do @ v.T
            ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
            dq = (ds @ k) / math.sqrt(d)
            dk = (ds.T @ q) / math.sqrt(d)
            dqkv[rows, h * d:(h + 1) * d] = dq
            dqkv[rows, H + h * d:H + (h + 1) * d] = dk
            dqkv[rows, 2 * H + h * d:2 * H + (h + 1) * d] = dv
    return dqkv


# ------------------------------------------------------------------ layer

def layer_fwd(arch, p, x, B, S, n_h, eps=1e-5):
    """One layer forward.  x [B*S, H] float64.  Returns (y, cache)."""
    x = np.asarray(x, dtype=np.float64)
    c = {"x": x}
    if arch == 0:
        attn_in = x
    else:
        attn_in, c["ln1"] = layernorm_fwd(x, p["g1"], p["be1"], eps)
    c["attn_in"] = attn_in
    qkv = attn_in @ p["Wqkv"] + p["bqkv"]
    ctx, probs = attention_fwd(qkv, B, S, n_h, causal=(arch == 1))
    a = ctx @ p["Wo"] + p["bo"]
    c.update(qkv=qkv, ctx=ctx, probs=probs)
    r1 = x + a
    if arch == 0:
        ffn_in, c["ln1"] = layernorm_fwd(r1, p["g1"], p["be1"], eps)
    else:
        ffn_in, c["ln2"] = layernorm_fwd(r1, p["g2"], p["be2"], eps)
    c["ffn_in"] = ffn_in
    h = ffn_in @ p["W1"] + p["b1"]
    g = gelu(h)
    f = g @ p["W2"] + p["b2"]
    c.update(h=h, g=g)
    if arch == 0:
        r2 = ffn_in + f
        y, c["ln2"] = layernorm_fwd(r2, p["g2"], p["be2"], eps)
    else:
        y = r1 + f
    return y, c


def layer_bwd(arch, p, c, dy):
    """One layer backward.  Returns (dx, grads) with grads keyed like PARAM_NAMES."""
    dy = np.asarray(dy, dtype=np.float64)
    G = {}
    if arch == 0:
        dr2, G["g2"], G["be2"] = layernorm_bwd(dy, p["g2"], c["ln2"])
        df = dr2
        d_ffn_in = dr2.copy()            # residual branch r2 = ffn_in + f
    else:
        df = dy
        dr1 = dy.copy()                  # residual branch y = r1 + f
    G["b2"] = df.sum(axis=0)
    G["W2"] = c["g"].T @ df
    dg = df @ p["W2"].T
    dh = dg * gelu_grad(c["h"])
    G["b1"] = dh.sum(axis=0)
    G["W1"] = c["ffn_in"].T @ dh
    if arch == 0:
        d_ffn_in = d_ffn_in + dh @ p["W1"].T
        dr1, G["g1"], G["be1"] = layernorm_bwd(d_ffn_in, p["g1"], c["ln1"])
    else:
        dv = dh @ p["W1"].T
        t, G["g2"], G["be2"] = layernorm_bwd(dv, p["g2"], c["ln2"])
        dr1 = dr1 + t
    da = dr1
    dx = dr1.copy()                      # residual branch r1 = x + a
    G["bo"] = da.sum(axis=0)
    G["Wo"] = c["ctx"].T @ da
    dctx = da @ p["Wo"].T
    B, n_h, S, _ = c["probs"].shape
    dqkv = attention_bwd(dctx, c["qkv"], c["probs"], B, S, n_h)
    G["bqkv"] = dqkv.sum(axis=0)
    G["Wqkv"] = c["attn_in"].T @ dqkv
    d_attn_in = dqkv @ p["Wqkv"].T
    if arch == 0:
        dx = dx + d_attn_in
    else:
        t, G["g1"], G["be1"] = layernorm_bwd(d_attn_in, p["g1"], c["ln1"])
        dx = dx + t
    return dx, G


# ------------------------------------------------------------ layer stacks

def stack_fwd(arch, layers, x, B, S, n_h, eps=1e-5):
    """Forward through a list of layers; returns (y, [cache per layer])."""
    caches = []
    for p in layers:
        x, c = layer_fwd(arch, p, x, B, S, n_h, eps)
        caches.append(c)
    return x, caches


def stack_bwd(arch, layers, caches, dy):
    """Backward through the stack; returns (dx, [grads per layer])."""
    grads = [None] * len(layers)
    for i in reversed(range(len(layers))):
        dy, grads[i] = layer_bwd(arch, layers[i], caches[i], dy)
    return dy, grads
