"""Kernels of the model's two ends against the oracle (GPU only): embedding forward and its
deterministic gradient, softmax cross-entropy forward / backward, the ordered sum."""
import numpy as np
import pytest
import torch

from oracle import ends as E
from paper_2204_12013_amd import synth
from util import TOL, assert_close, rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def B():
    from paper_2204_12013_amd import binding
    return binding


def _dev_ids(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


@pytest.mark.parametrize("dtype,V,S,Bsz,H", [(0, 37, 5, 3, 8), (0, 300, 21, 3, 72), (1, 1000, 200, 4, 256),
                                             (1, 97, 64, 9, 328), (1, 50304, 128, 4, 1600)])
def test_embedding_forward_and_gradient(B, dtype, V, S, Bsz, H):
    rng = np.random.default_rng(V)
    T = S * Bsz
    r = lambda a: synth.round_to_storage(a, dtype)
    Etok, Epos = r(rng.normal(0, 0.5, (V, H))), r(rng.normal(0, 0.5, (S, H)))
    ids = synth.zipf_ids(rng, V, T)
    g = r(rng.normal(0, 1, (T, H)))
    p = {"E_tok": Etok.astype(np.float64), "E_pos": Epos.astype(np.float64)}
    want, cache = E.front_fwd(1, p, ids, S)
    wg = E.front_bwd(1, p, cache, g.astype(np.float64))
    d_tok, d_pos, d_ids, d_g = B.to_device(Etok, dtype), B.to_device(Epos, dtype), _dev_ids(ids), B.to_device(g, dtype)
    out = torch.empty(T, H, dtype=d_tok.dtype, device=DEV)
    B.bk_embedding_fwd(d_ids, d_tok, d_pos, out)
    tol = TOL[dtype]
    assert_close(B.to_host(out), want, (1e-7 if dtype == 0 else tol), "ends B.to_host(out)")
    # gradients accumulate onto what is there
    init_t = rng.normal(0, 1, (V, H)).astype(np.float32)
    init_p = rng.normal(0, 1, (S, H)).astype(np.float32)
    runs = []
    for _ in range(2):
        gt, gp = torch.from_numpy(init_t).to(DEV), torch.from_numpy(init_p).to(DEV)
        B.bk_embedding_bwd(d_ids, d_g, gt, gp)
        torch.cuda.synchronize()
        runs.append((gt, gp))
    assert torch.equal(runs[0][0], runs[1][0]) and torch.equal(runs[0][1], runs[1][1])     # no atomics
    got_t = runs[0][0].cpu().numpy().astype(np.float64) - init_t
    got_p = runs[0][1].cpu().numpy().astype(np.float64) - init_p
    assert_close(got_t, wg["E_tok"], 1e-5, "ends got_t")
    assert_close(got_p, wg["E_pos"], 1e-5, "ends got_p")
    untouched = np.setdiff1d(np.arange(V), ids)
    assert np.array_equal(runs[0][0].cpu().numpy()[untouched], init_t[untouched])


def test_ids_outside_the_vocabulary_are_clamped(B):
    V, S, H = 16, 4, 8
    Etok = torch.arange(V * H, dtype=torch.float32, device=DEV).view(V, H)
    Epos = torch.zeros(S, H, device=DEV)
    out = torch.empty(S, H, device=DEV)
    B.bk_embedding_fwd(_dev_ids([-5, 0, V + 3, V - 1]), Etok, Epos, out)
    assert torch.equal(out[0], Etok[0]) and torch.equal(out[2], Etok[V - 1]) and torch.equal(out[3], Etok[V - 1])
    for bad in (dict(H=12), dict(V=0)):
        kw = dict(H=H, V=V)
        kw.update(bad)
        assert B.lib.bk_embedding_fwd(0, S, S, kw["H"], kw["V"], B._ptr(_dev_ids([0] * S)), B._ptr(Etok), B._ptr(Epos),
                                      B._ptr(out), None) == B.E_ARG


@pytest.mark.parametrize("dtype,T,V", [(0, 7, 16), (0, 33, 1000), (1, 130, 2048), (1, 65, 30528)])
def test_softmax_cross_entropy(B, dtype, T, V):
    rng = np.random.default_rng(T + V)
    logits = synth.round_to_storage(rng.normal(0, 3.0, (T, V)), dtype)
    logits[0, :] = 0.0                                   # uniform row: loss log V
    labels = synth.zipf_ids(rng, V, T)
    # the oracle's back end with an identity head and no LayerNorm is the loss on the logits themselves
    eye = {"W_head": np.eye(V)} if V <= 2048 else None
    x = logits.astype(np.float64)
    if eye is not None:
        loss, tok, cache = E.back_fwd(0, eye, x, labels)
        dl, _ = E.back_bwd(0, eye, cache)
        lse = cache[3]
    else:                                                # same formulas row by row without the V x V head
        m = x.max(axis=1)
        lse = m + np.log(np.exp(x - m[:, None]).sum(axis=1))
        tok = lse - x[np.arange(T), labels]
        loss = tok.mean()
        dl = np.exp(x - lse[:, None])
        dl[np.arange(T), labels] -= 1.0
        dl /= T
    d_logits, d_labels = B.to_device(logits, dtype), _dev_ids(labels)
    d_lse = torch.empty(T, dtype=torch.float32, device=DEV)
    d_tok = torch.empty(T, dtype=torch.float32, device=DEV)
    d_loss = torch.empty(1, dtype=torch.float32, device=DEV)
    B.bk_softmax_xent_fwd(d_logits, d_labels, d_lse, d_tok)
    B.bk_ordered_sum(d_tok, 1.0 / T, d_loss)
    assert np.allclose(d_lse.cpu().numpy(), lse, rtol=0, atol=2e-5)
    assert np.allclose(d_tok.cpu().numpy(), tok, rtol=0, atol=2e-5)
    assert abs(d_tok[0].item() - np.log(V)) < 2e-6
    assert abs(d_loss.item() - loss) <= 1e-5 * max(1.0, abs(loss))
    d_dl = torch.empty_like(d_logits)
    B.bk_softmax_xent_bwd(d_logits, d_labels, d_lse, 1.0 / T, d_dl)
    assert_close(B.to_host(d_dl), dl, (1e-5 if dtype == 0 else TOL[dtype]), "ends B.to_host(d_dl)")
    B.bk_softmax_xent_bwd(d_logits, d_labels, d_lse, 1.0 / T, d_logits)      # in place
    assert torch.equal(d_logits, d_dl)


def test_ordered_sum_is_reproducible(B):
    rng = np.random.default_rng(5)
    for n in (1, 255, 256, 4097):
        x = rng.normal(0, 1, n).astype(np.float32)
        d = torch.from_numpy(x).to(DEV)
        outs = []
        for _ in range(2):
            o = torch.empty(1, dtype=torch.float32, device=DEV)
            B.bk_ordered_sum(d, 0.5, o)
            outs.append(o.item())
        assert outs[0] == outs[1]
        assert abs(outs[0] - 0.5 * x.astype(np.float64).sum()) <= 1e-5 * max(1.0, np.abs(x).sum())


def test_bad_arguments_are_rejected(B):
    t = torch.zeros(16, 16, device=DEV)
    lab = _dev_ids([0] * 16)
    f = torch.zeros(16, device=DEV)
    p = B._ptr
    assert B.lib.bk_softmax_xent_fwd(0, 16, 12, p(t), p(lab), p(f), p(f), None) == B.E_ARG          # V not a multiple of 8
    assert B.lib.bk_softmax_xent_fwd(0, 0, 16, p(t), p(lab), p(f), p(f), None) == B.E_ARG
    assert B.lib.bk_softmax_xent_fwd(0, 16, 16, None, p(lab), p(f), p(f), None) == B.E_ARG
    assert B.lib.bk_softmax_xent_bwd(2, 16, 16, p(t), p(lab), p(f), 1.0, p(t), None) == B.E_ARG      # unknown dtype
    assert B.lib.bk_embedding_bwd(0, 16, 5, 16, 16, p(lab), p(t), p(t), p(t), None) == B.E_ARG       # tokens not a multiple of seq
    assert B.lib.bk_ordered_sum(0, p(f), 1.0, p(f), None) == B.E_ARG
    assert B.lib.bk_ordered_sum(16, None, 1.0, p(f), None) == B.E_ARG
