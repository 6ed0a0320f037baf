"""Pins for oracle/layer.py: nothing here calls the HIP path.

Each pin is chosen so that a dropped term, a wrong sign, a transposed operand
or a wrong index in the oracle fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

from oracle import layer as L


def _rand_layer(rng, H, F, scale=0.3):
    p = {}
    for n, shp in L.param_shapes(H, F).items():
        p[n] = rng.standard_normal(shp) * scale
        if n in ("g1", "g2"):
            p[n] = p[n] + 1.0
    return p


# --------------------------------------------------------- finite differences

@pytest.mark.parametrize("arch", [0, 1])
@pytest.mark.parametrize("shape", [(8, 2, 16, 4, 1), (64, 2, 256, 16, 2)])
def test_gradients_match_central_differences(arch, shape):
    H, n_h, F, S, B = shape
    rng = np.random.default_rng(7 + arch)
    p = _rand_layer(rng, H, F, scale=0.3 if H == 8 else 0.05)
    x = rng.standard_normal((B * S, H))
    Gm = rng.standard_normal((B * S, H))

    def loss(pp, xx):
        y, _ = L.layer_fwd(arch, pp, xx, B, S, n_h)
        return float((y * Gm).sum())

    y, c = L.layer_fwd(arch, p, x, B, S, n_h)
    dx, G = L.layer_bwd(arch, p, c, Gm)
    h = 1e-5

    def fd_x(idx):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        return (loss(p, xp) - loss(p, xm)) / (2 * h)

    idxs = [tuple(i) for i in np.argwhere(np.ones_like(x))] if H == 8 else \
        [tuple(rng.integers(0, s) for s in x.shape) for _ in range(60)]
    scale = np.abs(dx).max()
    for idx in idxs:
        assert abs(fd_x(idx) - dx[idx]) <= 1e-6 * scale + 1e-9, ("x", idx)

    n_samples = 200 if H == 8 else 25
    for name in L.PARAM_NAMES:
        scale = np.abs(G[name]).max() + 1e-12
        flat_n = p[name].size
        picks = rng.choice(flat_n, size=min(n_samples, flat_n), replace=False)
        for f in picks:
            idx = np.unravel_index(f, p[name].shape)
            pp = {k: v.copy() for k, v in p.items()}
            pp[name][idx] += h
            lp = loss(pp, x)
            pp[name][idx] -= 2 * h
            lm = loss(pp, x)
            fd = (lp - lm) / (2 * h)
            assert abs(fd - G[name][idx]) <= 1e-6 * scale + 1e-9, (name, idx, fd, G[name][idx])


# ------------------------------------- independent implementation (autograd)

def _torch_layer(arch, p, x, B, S, n_h, eps):
    """The same layer in torch float64 ops; gradients come from autograd."""
    F_ = torch.nn.functional
    H = x.shape[1]
    d = H // n_h

    def attn(u):
        qkv = u @ p["Wqkv"] + p["bqkv"]
        q, k, v = [t.reshape(B, S, n_h, d).permute(0, 2, 1, 3) for t in qkv.split(H, dim=1)]
        s = q @ k.transpose(-1, -2) / math.sqrt(d)
        if arch == 1:
            s = s.masked_fill(~torch.tril(torch.ones(S, S, dtype=torch.bool)), float("-inf"))
        ctx = (torch.softmax(s, dim=-1) @ v).permute(0, 2, 1, 3).reshape(B * S, H)
        return ctx @ p["Wo"] + p["bo"]

    def ffn(v):
        return F_.gelu(v @ p["W1"] + p["b1"]) @ p["W2"] + p["b2"]

    ln1 = lambda t: F_.layer_norm(t, (H,), p["g1"], p["be1"], eps)
    ln2 = lambda t: F_.layer_norm(t, (H,), p["g2"], p["be2"], eps)
    if arch == 0:
        y1 = ln1(x + attn(x))
        return ln2(y1 + ffn(y1))
    x1 = x + attn(ln1(x))
    return x1 + ffn(ln2(x1))


@pytest.mark.parametrize("arch", [0, 1])
def test_matches_torch_float64_autograd(arch):
    H, n_h, F, S, B = 64, 4, 192, 24, 3
    rng = np.random.default_rng(11)
    p = _rand_layer(rng, H, F, scale=0.1)
    x = rng.standard_normal((B * S, H))
    Gm = rng.standard_normal((B * S, H))
    y, c = L.layer_fwd(arch, p, x, B, S, n_h, eps=1e-5)
    dx, G = L.layer_bwd(arch, p, c, Gm)

    tp = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    ty = _torch_layer(arch, tp, tx, B, S, n_h, 1e-5)
    (ty * torch.tensor(Gm)).sum().backward()

    def close(a, b):
        return np.abs(a - b).max() <= 1e-10 * max(1.0, np.abs(b).max())
    assert close(y, ty.detach().numpy())
    assert close(dx, tx.grad.numpy())
    for n in L.PARAM_NAMES:
        assert close(G[n], tp[n].grad.numpy()), n


# ------------------------------------------------------ structural invariants

def test_softmax_rows_sum_to_one_and_causal_mask():
    rng = np.random.default_rng(3)
    B, S, n_h, H = 2, 10, 2, 16
    qkv = rng.standard_normal((B * S, 3 * H))
    _, probs = L.attention_fwd(qkv, B, S, n_h, causal=False)
    assert np.allclose(probs.sum(-1), 1.0, atol=1e-13) and (probs > 0).all()
    _, probs = L.attention_fwd(qkv, B, S, n_h, causal=True)
    assert np.allclose(probs.sum(-1), 1.0, atol=1e-13)
    assert (np.triu(probs, k=1) == 0).all()


def test_causal_output_ignores_future_tokens_and_batches_are_independent():
    rng = np.random.default_rng(5)
    H, n_h, F, S, B = 16, 2, 32, 8, 2
    p = _rand_layer(rng, H, F)
    x = rng.standard_normal((B * S, H))
    y, _ = L.layer_fwd(1, p, x, B, S, n_h)
    x2 = x.copy()
    x2[5:S] += 1.0                       # perturb tokens 5.. of sample 0
    y2, _ = L.layer_fwd(1, p, x2, B, S, n_h)
    assert np.array_equal(y[:5], y2[:5])          # earlier tokens unchanged
    assert not np.allclose(y[5:S], y2[5:S])
    assert np.array_equal(y[S:], y2[S:])          # other sample unchanged
    # bidirectional encoder: every token of the sample does change
    ye, _ = L.layer_fwd(0, p, x, B, S, n_h)
    ye2, _ = L.layer_fwd(0, p, x2, B, S, n_h)
    assert not np.allclose(ye[:5], ye2[:5]) and np.array_equal(ye[S:], ye2[S:])


def test_layernorm_statistics_and_shift_invariance():
    rng = np.random.default_rng(9)
    r = rng.standard_normal((7, 32)) * 3 + 2
    out, _ = L.layernorm_fwd(r, np.ones(32), np.zeros(32), 0.0)
    assert np.allclose(out.mean(-1), 0, atol=1e-13) and np.allclose(out.var(-1), 1, atol=1e-12)
    out2, _ = L.layernorm_fwd(r + 5.0, np.ones(32), np.zeros(32), 0.0)
    assert np.allclose(out, out2, atol=1e-12)
    g, b = rng.standard_normal(32), rng.standard_normal(32)
    out3, _ = L.layernorm_fwd(r, g, b, 0.0)
    assert np.allclose(out3, out * g + b, atol=1e-12)


def test_post_ln_output_is_normalised_and_uniform_attention_special_case():
    rng = np.random.default_rng(13)
    H, n_h, F, S, B = 16, 2, 32, 6, 1
    p = _rand_layer(rng, H, F)
    p["g2"], p["be2"] = np.ones(H), np.zeros(H)
    x = rng.standard_normal((B * S, H))
    y, _ = L.layer_fwd(0, p, x, B, S, n_h, eps=0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-12) and np.allclose(y.var(-1), 1, atol=1e-10)
    # zero query/key weights: every score is 0, attention is the mean of values
    q = {k: v.copy() for k, v in p.items()}
    q["Wqkv"][:, :2 * H] = 0
    q["bqkv"][:2 * H] = 0
    _, c = L.layer_fwd(0, q, x, B, S, n_h)
    v = x @ q["Wqkv"][:, 2 * H:] + q["bqkv"][2 * H:]
    assert np.allclose(c["ctx"], np.broadcast_to(v.mean(0), v.shape), atol=1e-12)


def test_gelu_values_and_derivative():
    assert L.gelu(np.array([0.0]))[0] == 0.0
    assert abs(L.gelu(np.array([1.0]))[0] - 0.5 * (1 + math.erf(1 / math.sqrt(2)))) < 1e-15
    big = L.gelu(np.array([10.0, -10.0]))
    assert abs(big[0] - 10.0) < 1e-12 and abs(big[1]) < 1e-12
    h = np.linspace(-4, 4, 41)
    fd = (L.gelu(h + 1e-6) - L.gelu(h - 1e-6)) / 2e-6
    assert np.allclose(fd, L.gelu_grad(h), atol=1e-8)


def test_parameter_count_matches_published_model_sizes():
    """Section 1 quotes BERT-Large at 340M and GPT-2 at 1.5B parameters; the
    layer stacks alone (no embeddings) must come in just under those figures."""
    bert = 24 * L.layer_param_count(1024, 4096)
    gpt2 = 48 * L.layer_param_count(1600, 6400)
    assert L.layer_param_count(1024, 4096) == 12 * 1024 ** 2 + 13 * 1024
    assert 0.85 * 340e6 < bert < 340e6
    assert 0.95 * 1.5e9 < gpt2 < 1.5e9
    H, F = 8, 24
    flat = np.arange(L.layer_param_count(H, F), dtype=np.float64)
    named = L.unpack_layer(flat, H, F)
    assert np.array_equal(L.pack_layer(named, H, F), flat)
    assert named["Wqkv"][1, 2] == 3 * H + 2 and named["bo"][0] == 3 * H * H + 3 * H + H * H
