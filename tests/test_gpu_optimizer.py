"""The APPLY step (Adam) and the replica weight synchronisation on the GPU, against
oracle/optim.py and against the invariant they exist for: FRC stays exactly the
successor's forward from one iteration to the next (paper Section 5.1), also
through a failover."""
import numpy as np
import pytest
import torch

from oracle import layer as L
from oracle import optim as O
from oracle import schedule as S
from oracle import stage as St
from paper_2204_12013_amd import synth
from util import assert_close, oracle_layers, rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# the hyper-parameters cross the ABI as C floats: both sides get the float32 values
HP = {k: float(np.float32(v)) for k, v in dict(lr=6e-3, beta1=0.9, beta2=0.999, eps=1e-8).items()}


@pytest.fixture(scope="module")
def B():
    from paper_2204_12013_amd import binding
    return binding


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("n", [4, 1028, 256 * 1024 * 3 + 64])
def test_adam_kernel_matches_oracle(B, dtype, n):
    """Same gradients on both sides: the fp32 kernel must track the fp64 update to fp32 rounding,
    and the storage copy must be exactly the rounded master weights."""
    rng = np.random.default_rng(n + dtype)
    act = torch.bfloat16 if dtype == 1 else torch.float32
    w0 = synth.round_to_storage((rng.standard_normal(n) * 0.02).astype(np.float32), dtype)
    master = torch.from_numpy(w0.copy()).to(DEV)
    m, v = torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
    w = torch.empty(n, dtype=act, device=DEV)
    wr, mr, vr = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in range(1, 5):
        g = (rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 1, n)).astype(np.float32)
        if step == 2:
            g[::7] = 0.0                                   # zero gradients: the moments only decay
        B.bk_adam(torch.from_numpy(g).to(DEV), master, m, v, w, step, **HP)
        wr, mr, vr = O.adam_step(wr, g.astype(np.float64), mr, vr, step, **HP)
        torch.cuda.synchronize()
        assert_close(m.cpu().numpy(), mr, 1e-6, "optimizer first moment")
        assert_close(v.cpu().numpy(), vr, 1e-6, "optimizer second moment")
        assert np.abs(master.cpu().numpy() - wr).max() <= 1e-6 * HP["lr"] * 50 + 1e-7 * np.abs(wr).max()
        assert torch.equal(w, master.to(act))


def test_adam_rejects_bad_arguments(B):
    t = torch.zeros(8, device=DEV)
    with pytest.raises(B.BambooError):
        B.bk_adam(t, t, t, t, t, 0)                        # steps count from 1
    with pytest.raises(B.BambooError):
        B.bk_adam(t[:6], t[:6], t[:6], t[:6], t[:6], 1)    # not a multiple of 4


def _stage_pair(B, sc, adam=HP):
    from paper_2204_12013_amd.harness import StageHarness
    inp = synth.make_stage_inputs(sc)
    st = B.Stage(B.make_cfg(sc), B.to_device(inp["own_w"].reshape(-1), sc.dtype),
                 B.to_device(inp["shadow_w"].reshape(-1), sc.dtype))
    scs = sc.replace(n_own=sc.n_shadow, n_shadow=0, stage_id=sc.stage_id + 1)
    succ = B.Stage(B.make_cfg(scs, frc_enabled=False), B.to_device(inp["shadow_w"].reshape(-1), sc.dtype), None)
    st.stage_optimizer_init()
    succ.stage_optimizer_init()
    x = [B.to_device(inp["x"][k], sc.dtype) for k in range(sc.M)]
    gz = [B.to_device(inp["gz"][k], sc.dtype) for k in range(sc.M)]
    torch.cuda.synchronize()
    return inp, st, succ, StageHarness(st, x, gz, successor=succ, adam=adam)


def test_training_iterations_match_oracle_fp32():
    """Three iterations of the tiny fp32 workload with Adam and replica synchronisation: parameters
    of the stage and of its replica against the oracle run the same way."""
    from paper_2204_12013_amd import binding as B
    sc = synth.CONFIGS["tiny"]
    inp, st, succ, hz = _stage_pair(B, sc)
    own = oracle_layers(inp["own_w"], sc.hidden, sc.ffn)
    shadow = oracle_layers(inp["shadow_w"], sc.hidden, sc.ffn)
    successor = [{n: a.copy() for n, a in p.items()} for p in shadow]
    opt_own, opt_succ = O.AdamState(own), O.AdamState(successor)
    x = {k: inp["x"][k].astype(np.float64) for k in range(sc.M)}
    gz = {k: inp["gz"][k].astype(np.float64) for k in range(sc.M)}
    prog = st.stage_schedule()
    for it in range(3):
        hz.begin_iteration()
        hz.run(prog)
        hz.sync()
        sim = St.StageSim(sc.arch, own, shadow, sc.micro_batch, sc.seq, sc.heads, sc.P, sc.stage_id, sc.M, x, gz)
        sim.run(S.stage_program(sc.P, sc.stage_id, sc.M))
        opt_own.apply(own, sim.G_own, **HP)
        opt_succ.apply(successor, sim.G_succ, **HP)
        O.sync_replica(shadow, successor)
        for k in range(sc.M):
            assert torch.equal(hz.z_frc[k], hz.z_succ[k]), (it, k)        # FRC == successor's forward, bitwise
            assert_close(B.to_host(hz.z_frc[k]), sim.z_frc[k], 1e-4, "optimizer z_frc %s" % ((it, k),))
        assert torch.equal(st.shadow_w, succ.own_w) and torch.equal(st.shadow_opt, succ.own_opt)
        got = st.own_w.cpu().numpy().astype(np.float64).reshape(sc.n_own, -1)
        for l in range(sc.n_own):
            ref = L.pack_layer(own[l], sc.hidden, sc.ffn)
            # the fp32 bar (1e-4) on the tensor; per element 1e-3: Adam divides by the gradient's own magnitude,
            # so a weight whose gradient is at the level of the fp32 rounding noise may step the other way
            assert_close(got[l], ref, 1e-4, "optimizer weights %s" % ((it, l),), elem_tol=1e-3)
    assert hz.step == 3
    st.stage_destroy()
    succ.stage_destroy()


def test_update_after_failover_equals_the_lost_successors_update_bf16(B):
    """Iteration 1 trains normally; in iteration 2 the successor is lost at micro-batch 2.  The merged
    stage's APPLY must leave the replica layers exactly where the successor's own APPLY would have
    left them (same gradients bitwise, same synchronised optimizer state), and the own layers where
    a failure-free run leaves them."""
    from paper_2204_12013_amd.harness import split_at_failure
    sc = synth.StageConfig("opt_b0", 0, 1, 256, 4, 1024, 64, 2, 2, 2, 4, 1, 5, 21)
    runs = []
    for fail in (False, True):
        inp, st, succ, hz = _stage_pair(B, sc)
        prog = st.stage_schedule()
        hz.begin_iteration()
        hz.run(prog)
        hz.sync()
        hz.begin_iteration()
        if not fail:
            hz.run(prog)
        else:
            hz.run(split_at_failure(prog, 2))
            succ.stage_sync()
            succ.own_g.zero_()
            hz.succ_dead = True
            hz.run(st.failover_merge(2))
        hz.sync()
        runs.append((st, succ, hz))
    (st0, succ0, hz0), (st1, succ1, hz1) = runs
    assert hz0.step == 2 and hz1.step == 2
    assert torch.equal(st1.own_w, st0.own_w)
    assert torch.equal(st1.shadow_w, succ0.own_w)            # the victim's layers, updated by the shadow
    assert torch.equal(st1.shadow_opt, succ0.own_opt)
    assert not torch.equal(st1.shadow_w, B.to_device(synth.make_stage_inputs(sc)["shadow_w"].reshape(-1), sc.dtype))
    for s_ in (st0, succ0, st1, succ1):
        s_.stage_destroy()


def test_optimizer_misuse_is_rejected(B):
    sc = synth.CONFIGS["tiny"]
    inp = synth.make_stage_inputs(sc)
    st = B.Stage(B.make_cfg(sc), B.to_device(inp["own_w"].reshape(-1), sc.dtype),
                 B.to_device(inp["shadow_w"].reshape(-1), sc.dtype))
    with pytest.raises(B.BambooError) as e:
        st.stage_apply(1)                                    # no optimizer state yet
    assert e.value.status == B.E_STATE
    st.stage_optimizer_init()
    with pytest.raises(B.BambooError):
        st.stage_apply(0)
    with pytest.raises(B.BambooError):
        st.stage_apply(1, beta1=1.5)
    st.stage_apply(1)
    st.stage_sync_replica(st.shadow_w)                       # weights only is allowed
    st.stage_sync()
    st.stage_destroy()
