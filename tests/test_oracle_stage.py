"""Pins for oracle/stage.py: the paper's two invariants, by brute force on tiny
pipelines (no HIP path involved).

Section 5.1: FRC on node n is exactly FNC of node n+1.
Sections 1, 5.2: after a preemption no computation is wasted and the lost
gradients are recomputed, so the iteration ends with the gradients of the
failure-free run.
"""
import itertools

import numpy as np
import pytest

from oracle import layer as L
from oracle import schedule as S
from oracle import stage as St


def _layers(rng, n, H, F):
    out = []
    for _ in range(n):
        p = {}
        for name, shp in L.param_shapes(H, F).items():
            p[name] = rng.standard_normal(shp) * 0.2 + (1.0 if name in ("g1", "g2") else 0.0)
        out.append(p)
    return out


def _setup(arch, P, s, M, n_own=1, n_shadow=1, seed=0):
    H, n_h, F, S_len, B = 8, 2, 16, 4, 1
    rng = np.random.default_rng(seed)
    own, shadow = _layers(rng, n_own, H, F), _layers(rng, n_shadow, H, F)
    x = {k: rng.standard_normal((B * S_len, H)) for k in range(M)}
    gz = {k: rng.standard_normal((B * S_len, H)) for k in range(M)}
    return (arch, own, shadow, B, S_len, n_h, P, s, M, x, gz)


@pytest.mark.parametrize("arch", [0, 1])
def test_frc_equals_successor_forward(arch):
    args = _setup(arch, 4, 1, 5, n_own=2, n_shadow=2)
    sim = St.run_no_failure(*args)
    for k in range(5):
        assert np.array_equal(sim.z_frc[k], sim.z_succ[k])
    assert all(not sim.own_stash for _ in [0])
    assert sorted(sim.shadow_stash) == list(range(5))       # FRC stash kept for the whole iteration
    # FRC off: same own results, nothing stashed
    sim2 = St.run_no_failure(*args, frc=False)
    assert not sim2.shadow_stash and not sim2.z_frc
    for k in range(5):
        assert np.array_equal(sim.gx[k], sim2.gx[k])


def test_stage_equals_one_deep_stack():
    """Own + shadow layers chained by the stage give what a single stack of all
    the layers gives (forward output and input gradient)."""
    arch, own, shadow, B, S_len, n_h, P, s, M, x, gz = _setup(1, 3, 0, 2, n_own=2, n_shadow=1)
    sim = St.run_no_failure(arch, own, shadow, B, S_len, n_h, P, s, M, x, gz)
    for k in range(M):
        z, caches = L.stack_fwd(arch, own + shadow, x[k], B, S_len, n_h)
        gx, grads = L.stack_bwd(arch, own + shadow, caches, gz[k])
        assert np.allclose(z, sim.z_frc[k], atol=1e-13)
        assert np.allclose(gx, sim.gx[k], atol=1e-13)


def test_failover_reproduces_failure_free_gradients_brute_force():
    n_cases = 0
    for arch in (0, 1):
        for P, M in itertools.product(range(2, 5), range(1, 6)):
            for s in range(P - 1):
                args = _setup(arch, P, s, M, seed=P * 10 + M)
                ref = St.run_no_failure(*args)
                for k_fail in range(M):
                    sim = St.run_with_failure(*args, k_fail)
                    n_cases += 1
                    assert sim.G_succ is None
                    for a, b in zip(sim.G_own, ref.G_own):
                        for n in L.PARAM_NAMES:
                            assert np.array_equal(a[n], b[n])
                    for a, b in zip(sim.G_shadow, ref.G_succ):
                        for n in L.PARAM_NAMES:
                            assert np.array_equal(a[n], b[n]), (P, M, s, k_fail, n)
                    for k in range(M):
                        assert np.array_equal(sim.gx[k], ref.gx[k])
                        assert np.array_equal(sim.z_frc[k], ref.z_succ[k])
                    assert not sim.own_stash and not sim.shadow_stash
                    # the replayed BRCs reproduce the g_y the victim had sent
                    for k, gy in getattr(sim, "gy_replay", {}).items():
                        assert np.array_equal(gy, ref.gy[k])
    assert n_cases > 100


def test_too_small_own_stash_is_detected():
    """The executor refuses to overwrite a live slot, so a capacity below the
    peak in-flight count cannot go unnoticed."""
    args = _setup(0, 4, 0, 6)
    sim = St.StageSim(*args)
    sim.C_own = 3                                   # stage 0 of 4 needs 4
    prog = [(op, lane, k, (k % 3 if op in (S.FWD, S.BWD) else a))
            for op, lane, k, a in S.stage_program(4, 0, 6)]
    with pytest.raises(AssertionError):
        sim.run(prog)


def test_record_index():
    assert St.stash_record_index(0, 0, 6) == 0
    assert St.stash_record_index(2, 3, 6) == 15


@pytest.mark.parametrize("rc", [S.LFLB, S.EFLB, S.EFEB])
def test_every_rc_variant_recovers_the_failure_free_gradients(rc):
    """Section 7.4 compares lazy/eager FRC and BRC: whatever is computed eagerly, a preemption must
    end with the gradients of the failure-free run (brute force over tiny pipelines, every k_fail)."""
    for P, s, M in [(3, 0, 4), (4, 1, 5), (2, 0, 3)]:
        args = _setup(0, P, s, M, seed=P * 10 + M)
        ref = St.run_no_failure(*args)
        for k_fail in range(M):
            sim = St.run_with_failure(*args, k_fail, rc=rc)
            for l in range(len(ref.G_own)):
                for n in L.PARAM_NAMES:
                    assert np.array_equal(sim.G_own[l][n], ref.G_own[l][n]), (P, s, M, k_fail, n)
                    assert np.array_equal(sim.G_shadow[l][n], ref.G_succ[l][n]), (P, s, M, k_fail, n)
            for k in range(M):
                assert np.array_equal(sim.gx[k], ref.gx[k])
                assert np.array_equal(sim.z_frc[k], ref.z_succ[k])
            assert not sim.own_stash and not sim.shadow_stash


def test_eager_brc_without_failure_reproduces_the_successors_gradients():
    args = _setup(1, 4, 1, 5, n_own=2, n_shadow=2)
    sim = St.run_no_failure(*args, rc=S.EFEB)
    for l in range(2):
        for n in L.PARAM_NAMES:
            assert np.array_equal(sim.G_shadow[l][n], sim.G_succ[l][n])
    assert not sim.shadow_stash                                 # every FRC stash was consumed by its BRC
    lazy = St.run_no_failure(*args, rc=S.LFLB)
    assert not lazy.z_frc and not lazy.shadow_stash
    for k in range(5):
        assert np.array_equal(lazy.gx[k], sim.gx[k])


def test_wrap_around_failover_rebuilds_the_first_stage_gradients():
    """Section 5.1 for the last node: whatever micro-batch the failure falls on, running the wrap-around
    failover schedule gives the last stage's own gradients (layers and head) of the failure-free program
    and, in the replica, exactly what the first stage would have accumulated (layers and embedding)."""
    from oracle import ends as E
    rng = np.random.default_rng(21)
    arch, H, F, n_h, Bsz, S_len, V, P, M = 1, 8, 16, 2, 2, 3, 13, 3, 4
    T = Bsz * S_len
    mk = lambda: L.unpack_layer(rng.normal(0, 0.3, L.layer_param_count(H, F)), H, F)
    own, shadow = [mk()], [mk(), mk()]
    front = E.unpack_front(rng.normal(0, 0.3, E.front_param_count(arch, V, S_len, H)), arch, V, S_len, H)
    back = E.unpack_back(rng.normal(0, 0.3, E.back_param_count(arch, V, H)), arch, V, H)
    x = {k: rng.normal(size=(T, H)) for k in range(M)}
    g1 = {k: rng.normal(size=(T, H)) for k in range(M)}
    ids = {k: rng.integers(0, V, T) for k in range(M)}
    labels = {k: rng.integers(0, V, T) for k in range(M)}
    args = (arch, own, back, shadow, front, Bsz, S_len, n_h, P, M, x, labels, ids, g1)
    ref = St.WrapStageSim(*args).run(S.stage_program(P, P - 1, M))
    Gv, Gfv, zv = St.wrap_first_stage_reference(arch, shadow, front, Bsz, S_len, n_h, M, ids, g1)
    for k in range(M):
        np.testing.assert_array_equal(ref.z_frc[k], zv[k])          # FRC is the first stage's forward
    for k_fail, rc in itertools.product(range(M), (S.EFLB, S.LFLB)):
        sim = St.WrapStageSim(*args)
        sim.run(S.prefix_until_failure(P, P - 1, M, k_fail, rc=rc))
        assert rc == S.EFLB or not sim.shadow_stash              # the lazy variant has run nothing redundant
        sim.run(S.wrap_failover_program(P, M, k_fail, rc=rc))
        assert not sim.own_stash and not sim.shadow_stash
        for k in range(M):
            np.testing.assert_array_equal(sim.z_frc[k], zv[k])
        for a, b in zip(sim.G_own, ref.G_own):
            for n in L.PARAM_NAMES:
                np.testing.assert_allclose(a[n], b[n], rtol=0, atol=1e-12)
        for n in ref.G_back:
            np.testing.assert_allclose(sim.G_back[n], ref.G_back[n], rtol=0, atol=1e-12)
        for a, b in zip(sim.G_shadow, Gv):
            for n in L.PARAM_NAMES:
                np.testing.assert_allclose(a[n], b[n], rtol=0, atol=1e-12)
        for n in Gfv:
            np.testing.assert_allclose(sim.G_front[n], Gfv[n], rtol=0, atol=1e-12)
        assert sim.loss == ref.loss


def test_merged_iteration_is_one_deep_stage():
    """Section 5.2: until the pipeline is reconfigured the shadow node executes all of the victim's
    instructions.  A whole iteration of the merged program must therefore be an ordinary stage of
    own + replica layers: outputs, input gradients and both gradient sets equal one deep stack's."""
    for arch, P, s, M in [(0, 4, 1, 5), (1, 3, 0, 4), (0, 2, 0, 3), (1, 5, 3, 6)]:
        arch, own, shadow, B, S_len, n_h, P, s, M, x, gz = _setup(arch, P, s, M, n_own=2, n_shadow=2, seed=P + M)
        sim = St.StageSim(arch, own, shadow, B, S_len, n_h, P, s, M, x, gz)
        sim.preempt_successor()
        sim.run(S.merged_program(P, s, M))
        assert not sim.own_stash and not sim.shadow_stash
        G = None
        for k in range(M):
            z, caches = L.stack_fwd(arch, own + shadow, x[k], B, S_len, n_h)
            gx, grads = L.stack_bwd(arch, own + shadow, caches, gz[k])
            np.testing.assert_allclose(sim.z_frc[k], z, rtol=0, atol=1e-13)
            np.testing.assert_allclose(sim.gx[k], gx, rtol=0, atol=1e-13)
            G = grads if G is None else [{n: a[n] + b[n] for n in L.PARAM_NAMES} for a, b in zip(G, grads)]
        for got, want in zip(sim.G_own + sim.G_shadow, G):
            for n in L.PARAM_NAMES:
                np.testing.assert_allclose(got[n], want[n], rtol=0, atol=1e-12)
        # and it is what the failure-free pair of stages accumulates (same order of additions: bitwise)
        ref = St.run_no_failure(arch, own, shadow, B, S_len, n_h, P, s, M, x, gz)
        for a, b in zip(sim.G_shadow, ref.G_succ):
            for n in L.PARAM_NAMES:
                assert np.array_equal(a[n], b[n])
        for a, b in zip(sim.G_own, ref.G_own):
            for n in L.PARAM_NAMES:
                assert np.array_equal(a[n], b[n])


def _dp_setup(arch, M, seed=0, same_weights=False):
    H, n_h, F, S_len, B = 8, 2, 16, 4, 1
    rng = np.random.default_rng(seed)
    own = _layers(rng, 2, H, F)
    replica = [dict(p) for p in own] if same_weights else _layers(rng, 2, H, F)
    mk = lambda: {k: rng.standard_normal((B * S_len, H)) for k in range(M)}
    return (arch, own, replica, B, S_len, n_h, M, mk(), mk(), mk(), mk())


def test_data_parallel_eager_frc_is_over_batching():
    """Section 5.2, pure data parallelism: eager FRC amounts to the node processing its own minibatch
    plus a redundant one.  With equal parameters (a synchronous job) the node's own gradient plus the
    replica's, after BRC, must be the gradient of ONE pass over the two minibatches put together."""
    for arch in (0, 1):
        M = 3
        args = _dp_setup(arch, M, seed=5 + arch, same_weights=True)
        arch, own, replica, B, S_len, n_h, M, x, g, xn, gn = args
        sim = St.DataParallelSim(*args).run(S.merged_program(1, 0, M))
        G = None
        for k in range(M):
            both_x, both_g = np.concatenate([x[k], xn[k]]), np.concatenate([g[k], gn[k]])
            _, caches = L.stack_fwd(arch, own, both_x, 2 * B, S_len, n_h)
            _, grads = L.stack_bwd(arch, own, caches, both_g)
            G = grads if G is None else [{n: a[n] + b[n] for n in L.PARAM_NAMES} for a, b in zip(G, grads)]
        for l in range(len(own)):
            for n in L.PARAM_NAMES:
                np.testing.assert_allclose(sim.G_own[l][n] + sim.G_shadow[l][n], G[l][n], rtol=0, atol=1e-11)


@pytest.mark.parametrize("rc", [S.LFLB, S.EFLB])
def test_data_parallel_failover_rebuilds_the_lost_nodes_gradient(rc):
    """Whatever micro-batch the loss of the other node falls on, the iteration ends with this node's own
    gradient and, in the replica, exactly the gradient the lost node would have contributed to the
    all-reduce (brute force, every k_fail; different parameter values in the replica so that a mix-up
    of the two parameter sets cannot cancel)."""
    M = 4
    args = _dp_setup(1, M, seed=9)
    arch, own, replica, B, S_len, n_h, M, x, g, xn, gn = args
    ref = St.DataParallelSim(*args)
    ref.run(S.stage_program(1, 0, M, rc=rc))
    z_neigh = [ref._neighbour_step(k) for k in range(M)]        # what the other node computes itself
    assert not any(op in (S.SEND_ACT, S.RECV_ACT, S.SEND_GRAD, S.RECV_GRAD)
                   for op, _, _, _ in S.stage_program(1, 0, M, rc=rc))
    for k_fail in range(M):
        sim = St.DataParallelSim(*args)
        sim.run(S.prefix_until_failure(1, 0, M, k_fail, rc=rc))
        sim.preempt_neighbour()
        prog = S.failover_program(1, 0, M, k_fail, rc=rc, data_parallel=True)
        sim.run(prog)
        assert not any(op in (S.SEND_ACT, S.RECV_ACT, S.SEND_GRAD, S.RECV_GRAD) for op, _, _, _ in prog)
        assert sorted(k for op, _, k, _ in prog if op == S.BRC) == list(range(M))      # every micro-batch once
        assert not sim.own_stash and not sim.shadow_stash
        for l in range(len(own)):
            for n in L.PARAM_NAMES:
                assert np.array_equal(sim.G_own[l][n], ref.G_own[l][n])
                assert np.array_equal(sim.G_shadow[l][n], ref.G_neigh[l][n]), (k_fail, l, n)
        for k in range(M):
            assert np.array_equal(sim.z_frc[k], z_neigh[k])
            assert np.array_equal(sim.gx[k], ref.gx[k])


def test_wrap_merged_iteration_equals_the_two_failure_free_stages():
    """A whole iteration of the last stage after it has taken over the first (Section 5.2: the shadow executes
    all of the victim's instructions): own side as in the failure-free program, replica side what the first
    stage itself would accumulate."""
    from oracle import ends as E
    rng = np.random.default_rng(22)
    arch, H, F, n_h, Bsz, S_len, V, P, M = 0, 8, 16, 2, 1, 4, 11, 4, 5
    T = Bsz * S_len
    mk = lambda: L.unpack_layer(rng.normal(0, 0.3, L.layer_param_count(H, F)), H, F)
    own, shadow = [mk(), mk()], [mk()]
    front = E.unpack_front(rng.normal(0, 0.3, E.front_param_count(arch, V, S_len, H)), arch, V, S_len, H)
    back = E.unpack_back(rng.normal(0, 0.3, E.back_param_count(arch, V, H)), arch, V, H)
    x = {k: rng.normal(size=(T, H)) for k in range(M)}
    g1 = {k: rng.normal(size=(T, H)) for k in range(M)}
    ids = {k: rng.integers(0, V, T) for k in range(M)}
    labels = {k: rng.integers(0, V, T) for k in range(M)}
    args = (arch, own, back, shadow, front, Bsz, S_len, n_h, P, M, x, labels, ids, g1)
    ref = St.WrapStageSim(*args).run(S.stage_program(P, P - 1, M))
    Gv, Gfv, zv = St.wrap_first_stage_reference(arch, shadow, front, Bsz, S_len, n_h, M, ids, g1)
    sim = St.WrapStageSim(*args).run(S.wrap_merged_program(P, M))
    assert not sim.own_stash and not sim.shadow_stash and sim.loss == ref.loss
    for a, b in zip(sim.G_own, ref.G_own):
        for n in L.PARAM_NAMES:
            np.testing.assert_array_equal(a[n], b[n])
    for a, b in zip(sim.G_shadow, Gv):
        for n in L.PARAM_NAMES:
            np.testing.assert_allclose(a[n], b[n], rtol=0, atol=1e-12)
    for n in Gfv:
        np.testing.assert_allclose(sim.G_front[n], Gfv[n], rtol=0, atol=1e-12)
