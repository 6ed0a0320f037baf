"""Pins of the oracle's model ends (token/position embedding at the front, LM head + mean
cross-entropy at the back) against things other than itself: torch's CPU autograd over its own
embedding / layer_norm / cross_entropy routines, central differences, closed forms."""
import numpy as np
import pytest
import torch

from oracle import ends as E


def _params(arch, V, S, H, rng):
    f = rng.normal(0, 0.3, E.front_param_count(arch, V, S, H))
    b = rng.normal(0, 0.3, E.back_param_count(arch, V, H))
    if arch == 0:
        f[(V + S) * H:(V + S) * H + H] += 1.0
    else:
        b[:H] += 1.0
    return f, b


@pytest.mark.parametrize("arch", [0, 1])
def test_front_and_back_match_torch_autograd(arch):
    rng = np.random.default_rng(3 + arch)
    V, S, H, Bsz = 37, 5, 12, 3
    T = S * Bsz
    f, b = _params(arch, V, S, H, rng)
    ids = rng.integers(0, V, T)
    ids[4] = ids[1]                                     # a token that occurs twice
    labels = rng.integers(0, V, T)
    pf, pb = E.unpack_front(f, arch, V, S, H), E.unpack_back(b, arch, V, H)
    x0, cf = E.front_fwd(arch, pf, ids, S)
    loss, tok, cb = E.back_fwd(arch, pb, x0, labels)    # back applied straight to the front's output
    dy, gb = E.back_bwd(arch, pb, cb)
    gf = E.front_bwd(arch, pf, cf, dy)

    tf = torch.tensor(f, dtype=torch.float64, requires_grad=True)
    tb = torch.tensor(b, dtype=torch.float64, requires_grad=True)
    Etok, Epos = tf[:V * H].view(V, H), tf[V * H:(V + S) * H].view(S, H)
    e = torch.nn.functional.embedding(torch.tensor(ids), Etok) + Epos.repeat(Bsz, 1)
    if arch == 0:
        e = torch.nn.functional.layer_norm(e, (H,), tf[(V + S) * H:(V + S) * H + H], tf[(V + S) * H + H:], 1e-5)
    h = e
    off = 0
    if arch == 1:
        h = torch.nn.functional.layer_norm(e, (H,), tb[:H], tb[H:2 * H], 1e-5)
        off = 2 * H
    logits = h @ tb[off:].view(H, V)
    tl = torch.nn.functional.cross_entropy(logits, torch.tensor(labels))
    tl.backward()
    assert abs(loss - tl.item()) < 1e-12
    np.testing.assert_allclose(x0, e.detach().numpy(), rtol=0, atol=1e-12)
    want_f = E.unpack_front(tf.grad.numpy(), arch, V, S, H)
    want_b = E.unpack_back(tb.grad.numpy(), arch, V, H)
    for k in want_f:
        np.testing.assert_allclose(gf[k], want_f[k], rtol=0, atol=1e-12, err_msg=k)
    for k in want_b:
        np.testing.assert_allclose(gb[k], want_b[k], rtol=0, atol=1e-12, err_msg=k)


def test_closed_forms():
    rng = np.random.default_rng(0)
    V, S, H, T = 11, 4, 6, 8
    # a zero head gives uniform predictions: loss = log V, and each gradient row of the logits sums to 0
    pb = {"W_head": np.zeros((H, V))}
    y = rng.normal(size=(T, H))
    labels = rng.integers(0, V, T)
    loss, tok, cache = E.back_fwd(0, pb, y, labels)
    assert abs(loss - np.log(V)) < 1e-14 and np.allclose(tok, np.log(V))
    dy, g = E.back_bwd(0, pb, cache)
    assert np.allclose(dy, 0.0)
    # dW_head[:, v] = sum_t y[t] (1/V - [labels[t] = v]) / T
    want = np.zeros((H, V))
    for t in range(T):
        for v in range(V):
            want[:, v] += y[t] * (1.0 / V - (labels[t] == v)) / T
    np.testing.assert_allclose(g["W_head"], want, atol=1e-14)
    np.testing.assert_allclose(g["W_head"].sum(axis=1), 0.0, atol=1e-14)
    # a head that puts a large margin on the label: loss -> 0
    Wbig = np.zeros((H, V))
    y1 = np.zeros((T, H)); y1[:, 0] = 1.0
    Wbig[0, 3] = 50.0
    loss, _, _ = E.back_fwd(0, {"W_head": Wbig}, y1, np.full(T, 3))
    assert 0 <= loss < 1e-20 + 11 * np.exp(-50.0)
    # every token the same id: that row of the table collects the sum of all rows of the gradient
    pf = {"E_tok": rng.normal(size=(V, H)), "E_pos": rng.normal(size=(S, H))}
    ids = np.full(T, 7)
    x0, cf = E.front_fwd(1, pf, ids, S)
    np.testing.assert_allclose(x0[5], pf["E_tok"][7] + pf["E_pos"][1], atol=0)
    d = rng.normal(size=(T, H))
    g = E.front_bwd(1, pf, cf, d)
    np.testing.assert_allclose(g["E_tok"][7], d.sum(axis=0), atol=1e-14)
    assert np.count_nonzero(np.delete(g["E_tok"], 7, axis=0)) == 0
    np.testing.assert_allclose(g["E_pos"][2], d[2] + d[6], atol=1e-14)


@pytest.mark.parametrize("arch", [0, 1])
def test_central_differences(arch):
    rng = np.random.default_rng(11)
    V, S, H, T = 9, 3, 4, 6
    f, b = _params(arch, V, S, H, rng)
    ids = np.array([2, 5, 2, 0, 5, 2])
    labels = rng.integers(0, V, T)

    def loss_of(f_, b_):
        x0, _ = E.front_fwd(arch, E.unpack_front(f_, arch, V, S, H), ids, S)
        return E.back_fwd(arch, E.unpack_back(b_, arch, V, H), x0, labels)[0]
    pf, pb = E.unpack_front(f, arch, V, S, H), E.unpack_back(b, arch, V, H)
    x0, cf = E.front_fwd(arch, pf, ids, S)
    _, _, cb = E.back_fwd(arch, pb, x0, labels)
    dy, gb = E.back_bwd(arch, pb, cb)
    gf = E.front_bwd(arch, pf, cf, dy)
    flat_f = np.concatenate([gf["E_tok"].ravel(), gf["E_pos"].ravel()] + ([gf["g_e"], gf["b_e"]] if arch == 0 else []))
    flat_b = np.concatenate(([gb["g_f"], gb["b_f"]] if arch == 1 else []) + [gb["W_head"].ravel()])
    h = 1e-6
    for i in rng.choice(f.size, 25, replace=False):
        d = np.zeros_like(f); d[i] = h
        num = (loss_of(f + d, b) - loss_of(f - d, b)) / (2 * h)
        assert abs(num - flat_f[i]) < 1e-8, ("front", i)
    for i in rng.choice(b.size, 25, replace=False):
        d = np.zeros_like(b); d[i] = h
        num = (loss_of(f, b + d) - loss_of(f, b - d)) / (2 * h)
        assert abs(num - flat_b[i]) < 1e-8, ("back", i)
