"""The two ends of the model in float64 (oracle; test infrastructure).

Section 5.1: the first node's layers are replicated on the last node, which
fetches the input samples itself to run redundant computation for the first
node.  So the wrap-around stage works on what the middle stages never see:
token ids at the front of the model and the loss at its back.  The paper does
not spell these out; they are the textbook ends of the models it trains
(Section 7, Table 1: BERT-Large, GPT-2), written here as the plain formulas:

  front (first node)   e[t] = E_tok[ids[t]] + E_pos[t mod S]
                       arch 0 (post-LN encoder): x0 = LayerNorm(e; g_e, b_e)
                       arch 1 (pre-LN decoder):  x0 = e
  back (last node)     arch 0: hf = y
                       arch 1: hf = LayerNorm(y; g_f, b_f)      (final LayerNorm)
                       logits = hf W_head          W_head [H, V]
                       loss   = mean over the T tokens of
                                log(sum_v exp(logits[t, v])) - logits[t, labels[t]]

Flat parameter layouts (gradients use the same):
  front: E_tok [V,H] | E_pos [S,H] | g_e [H] | b_e [H]      (the last two only for arch 0)
  back:  g_f [H] | b_f [H] | W_head [H,V]                   (the first two only for arch 1)
"""
import numpy as np

from . import layer as L


def front_param_count(arch, V, S, H):
    return V * H + S * H + (2 * H if arch == 0 else 0)


def back_param_count(arch, V, H):
    return (2 * H if arch == 1 else 0) + H * V


def unpack_front(flat, arch, V, S, H):
    flat = np.asarray(flat, dtype=np.float64)
    out = {"E_tok": flat[:V * H].reshape(V, H), "E_pos": flat[V * H:V * H + S * H].reshape(S, H)}
    if arch == 0:
        out["g_e"] = flat[(V + S) * H:(V + S) * H + H]
        out["b_e"] = flat[(V + S) * H + H:(V + S) * H + 2 * H]
    assert flat.size == front_param_count(arch, V, S, H)
    return out


def unpack_back(flat, arch, V, H):
    flat = np.asarray(flat, dtype=np.float64)
    out, off = {}, 0
    if arch == 1:
        out["g_f"], out["b_f"] = flat[:H], flat[H:2 * H]
        off = 2 * H
    out["W_head"] = flat[off:].reshape(H, V)
    assert flat.size == back_param_count(arch, V, H)
    return out


def front_fwd(arch, p, ids, S, eps=1e-5):
    """ids: int array [T], token t is position t mod S of sample t // S."""
    T = ids.shape[0]
    pos = np.arange(T) % S
    e = p["E_tok"][ids] + p["E_pos"][pos]
    if arch == 0:
        x0, ln = L.layernorm_fwd(e, p["g_e"], p["b_e"], eps)
        return x0, (ids, pos, ln)
    return e, (ids, pos, None)


def front_bwd(arch, p, cache, dx0):
    """Gradients of the front parameters from the gradient at the front's output."""
    ids, pos, ln = cache
    grads = {}
    de = dx0
    if arch == 0:
        de, grads["g_e"], grads["b_e"] = L.layernorm_bwd(dx0, p["g_e"], ln)
    grads["E_tok"] = np.zeros_like(p["E_tok"])
    grads["E_pos"] = np.zeros_like(p["E_pos"])
    for t in range(ids.shape[0]):            # rows that occur several times add up
        grads["E_tok"][ids[t]] += de[t]
        grads["E_pos"][pos[t]] += de[t]
    return grads


def back_fwd(arch, p, y, labels, eps=1e-5):
    """Returns (loss, per-token losses, cache)."""
    ln = None
    hf = y
    if arch == 1:
        hf, ln = L.layernorm_fwd(y, p["g_f"], p["b_f"], eps)
    logits = hf @ p["W_head"]
    m = logits.max(axis=-1, keepdims=True)
    lse = m[:, 0] + np.log(np.exp(logits - m).sum(axis=-1))
    tok = lse - logits[np.arange(labels.shape[0]), labels]
    return tok.mean(), tok, (hf, ln, logits, lse, labels)


def back_bwd(arch, p, cache, dloss=1.0):
    """Returns (gradient at the back's input y, parameter gradients)."""
    hf, ln, logits, lse, labels = cache
    T = labels.shape[0]
    dlogits = np.exp(logits - lse[:, None])
    dlogits[np.arange(T), labels] -= 1.0
    dlogits *= dloss / T
    grads = {"W_head": hf.T @ dlogits}
    dhf = dlogits @ p["W_head"].T
    if arch == 1:
        dy, grads["g_f"], grads["b_f"] = L.layernorm_bwd(dhf, p["g_f"], ln)
        return dy, grads
    return dhf, grads
