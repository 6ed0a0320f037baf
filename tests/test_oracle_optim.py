"""Pins for oracle/optim.py (no HIP path involved).

The Adam update is checked against things other than itself: torch.optim.Adam
(an independent library implementation, CPU float64), the closed form of the
first step, and two invariants."""
import numpy as np
import torch

from oracle import optim as O


def test_adam_matches_library_adam_over_several_steps():
    rng = np.random.default_rng(0)
    w0 = rng.standard_normal((7, 5))
    grads = [rng.standard_normal((7, 5)) * (10.0 ** rng.integers(-3, 2)) for _ in range(6)]
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.Adam([p], lr=6e-3, betas=(0.9, 0.999), eps=1e-8)
    for t, g in enumerate(grads, start=1):
        w, m, v = O.adam_step(w, g, m, v, t, 6e-3)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        assert np.allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-14), t


def test_first_step_closed_form():
    # after one step m_hat = g and v_hat = g^2, so the update is -lr * g / (|g| + eps)
    g = np.array([3.0, -0.5, 1e-3, -20.0])
    w, m, v = O.adam_step(np.zeros(4), g, np.zeros(4), np.zeros(4), 1, 6e-3)
    assert np.allclose(w, -6e-3 * g / (np.abs(g) + 1e-8), rtol=1e-13)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 0.001 * g * g)


def test_zero_gradient_leaves_fresh_parameters_alone_and_sign_follows_gradient():
    w0 = np.array([1.0, -2.0])
    w, m, v = O.adam_step(w0, np.zeros(2), np.zeros(2), np.zeros(2), 1, 6e-3)
    assert np.array_equal(w, w0) and not m.any() and not v.any()
    w, _, _ = O.adam_step(w0, np.array([5.0, -5.0]), np.zeros(2), np.zeros(2), 1, 6e-3)
    assert w[0] < w0[0] and w[1] > w0[1]


def test_state_object_and_replica_sync():
    rng = np.random.default_rng(1)
    succ = [{"a": rng.standard_normal(3), "b": rng.standard_normal((2, 2))}]
    shadow = [{k: x.copy() for k, x in succ[0].items()}]
    st = O.AdamState(succ)
    g = [{"a": rng.standard_normal(3), "b": rng.standard_normal((2, 2))}]
    before = succ[0]["a"].copy()
    st.apply(succ, g, 6e-3)
    assert st.step == 1 and not np.array_equal(succ[0]["a"], before)
    assert np.array_equal(shadow[0]["a"], before)            # the replica is stale until synchronised
    O.sync_replica(shadow, succ)
    assert all(np.array_equal(shadow[0][k], succ[0][k]) for k in succ[0])
    succ[0]["a"][0] += 1.0
    assert shadow[0]["a"][0] != succ[0]["a"][0]              # a copy, not an alias
