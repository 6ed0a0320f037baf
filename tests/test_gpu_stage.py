"""Parity of the whole stage with the oracle through the C ABI (GPU only):
FNC/BNC, eager FRC on the second lane, failover + lazy BRC.  Also the paper's
two invariants on the GPU itself, bitwise."""
import numpy as np
import pytest
import torch

from oracle import schedule as S
from oracle import stage as St
from paper_2204_12013_amd import synth
from util import TOL, assert_close, check_grads, oracle_layers, rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SMALL = {
    # the tiny workload of the table: fp32, 1 own + 1 shadow post-LN layer
    "tiny": synth.CONFIGS["tiny"],
    # ragged fp32 shapes, pre-LN causal, 2+2 layers, deeper pipeline
    "ragged_fp32_causal": synth.StageConfig("r32", 1, 0, 72, 3, 200, 21, 3, 2, 2, 4, 1, 5, 11),
    # bf16, post-LN, head size 64, several tiles with a ragged tail
    "bf16_post_ln": synth.StageConfig("b0", 0, 1, 256, 4, 1024, 200, 2, 2, 2, 4, 1, 5, 12),
    # bf16, pre-LN causal, head size 128
    "bf16_causal_d128": synth.StageConfig("b1", 1, 1, 256, 2, 768, 160, 1, 2, 2, 4, 2, 4, 13),
    # bf16, pre-LN causal, hidden not a multiple of 128 (GPT-2 1.5B style 25-head split scaled down)
    "bf16_causal_h320": synth.StageConfig("b2", 1, 1, 320, 5, 1280, 96, 2, 1, 2, 3, 0, 4, 14),
}


@pytest.fixture(scope="module")
def B():
    from paper_2204_12013_amd import binding
    return binding


def _build(B, sc, frc=True, with_successor=True):
    from paper_2204_12013_amd.harness import StageHarness
    inp = synth.make_stage_inputs(sc)
    cfg = B.make_cfg(sc, frc_enabled=frc)
    st = B.Stage(cfg, B.to_device(inp["own_w"].reshape(-1), sc.dtype), B.to_device(inp["shadow_w"].reshape(-1), sc.dtype))
    succ = None
    if with_successor:
        scs = sc.replace(n_own=sc.n_shadow, n_shadow=0, stage_id=sc.stage_id + 1)
        succ = B.Stage(B.make_cfg(scs, frc_enabled=False), B.to_device(inp["shadow_w"].reshape(-1), sc.dtype), None)
    x = [B.to_device(inp["x"][k], sc.dtype) for k in range(sc.M)]
    gz = [B.to_device(inp["gz"][k], sc.dtype) for k in range(sc.M)]
    torch.cuda.synchronize()
    return inp, st, StageHarness(st, x, gz, successor=succ)


def _oracle(sc, inp, k_fail=None):
    own = oracle_layers(inp["own_w"], sc.hidden, sc.ffn)
    shadow = oracle_layers(inp["shadow_w"], sc.hidden, sc.ffn)
    x = {k: inp["x"][k].astype(np.float64) for k in range(sc.M)}
    gz = {k: inp["gz"][k].astype(np.float64) for k in range(sc.M)}
    args = (sc.arch, own, shadow, sc.micro_batch, sc.seq, sc.heads, sc.P, sc.stage_id, sc.M, x, gz)
    return St.run_no_failure(*args) if k_fail is None else St.run_with_failure(*args, k_fail)


@pytest.mark.parametrize("name", list(SMALL))
def test_iteration_matches_oracle(B, name):
    sc = SMALL[name]
    tol = TOL[sc.dtype]
    inp, st, hz = _build(B, sc)
    prog = st.stage_schedule()
    assert prog == S.stage_program(sc.P, sc.stage_id, sc.M)
    hz.begin_iteration()
    hz.run(prog)
    hz.sync()
    ref = _oracle(sc, inp)
    for k in range(sc.M):
        assert_close(B.to_host(hz.y[k]), ref.y[k], tol, "stage B.to_host(hz.y[k]) %s" % (("y", k),))
        assert_close(B.to_host(hz.z_frc[k]), ref.z_frc[k], tol, "stage B.to_host(hz.z_frc[k]) %s" % (("z", k),))
        assert_close(B.to_host(hz.gy[k]), ref.gy[k], tol, "stage B.to_host(hz.gy[k]) %s" % (("gy", k),))
        assert_close(B.to_host(hz.gx[k]), ref.gx[k], tol, "stage B.to_host(hz.gx[k]) %s" % (("gx", k),))
        # Section 5.1: FRC is exactly the successor's forward -- bitwise on the GPU
        assert torch.equal(hz.z_frc[k], hz.z_succ[k])
    check_grads(st.own_g.cpu().numpy(), ref.G_own, sc.hidden, sc.ffn, tol, "own")
    check_grads(hz.succ.own_g.cpu().numpy(), ref.G_succ, sc.hidden, sc.ffn, tol, "successor")
    assert float(st.shadow_g.abs().max()) == 0.0          # lazy BRC: nothing ran
    st.stage_destroy()
    hz.succ.stage_destroy()


@pytest.mark.parametrize("name,k_fail", [("tiny", 1), ("tiny", 3), ("ragged_fp32_causal", 0),
                                         ("ragged_fp32_causal", 3), ("bf16_post_ln", 2), ("bf16_causal_d128", 1)])
def test_failover_matches_oracle_and_failure_free_run(B, name, k_fail):
    from paper_2204_12013_amd.harness import split_at_failure
    sc = SMALL[name]
    tol = TOL[sc.dtype]
    # failure-free run on the GPU
    inp, st0, hz0 = _build(B, sc)
    hz0.begin_iteration()
    hz0.run(st0.stage_schedule())
    hz0.sync()
    # run with the successor lost while handing over micro-batch k_fail
    _, st, hz = _build(B, sc)
    hz.begin_iteration()
    hz.run(split_at_failure(st.stage_schedule(), k_fail))
    hz.succ.stage_sync()
    hz.succ.own_g.zero_()            # the victim's accumulated gradients are gone
    hz.succ_dead = True
    merged = st.failover_merge(k_fail)
    assert merged == S.failover_program(sc.P, sc.stage_id, sc.M, k_fail)
    assert st.stage_schedule() == merged
    hz.run(merged)
    hz.sync()
    ref = _oracle(sc, inp, k_fail)
    check_grads(st.own_g.cpu().numpy(), ref.G_own, sc.hidden, sc.ffn, tol, "own")
    check_grads(st.shadow_g.cpu().numpy(), ref.G_shadow, sc.hidden, sc.ffn, tol, "shadow")
    for k in range(sc.M):
        assert_close(B.to_host(hz.gx[k]), ref.gx[k], tol, "stage B.to_host(hz.gx[k])")
        assert_close(B.to_host(hz.z_frc[k]), ref.z_frc[k], tol, "stage B.to_host(hz.z_frc[k])")
    # Sections 1 and 5.2: nothing is lost -- gradients equal the failure-free run's, bitwise
    assert torch.equal(st.own_g, st0.own_g)
    assert torch.equal(st.shadow_g, hz0.succ.own_g)
    for k in range(sc.M):
        assert torch.equal(hz.gx[k], hz0.gx[k])
        assert torch.equal(hz.z_frc[k], hz0.z_succ[k])
    for k, gy in hz.gy_replay.items():
        assert torch.equal(gy, hz0.gy[k])
    for s_ in (st0, st, hz0.succ, hz.succ):
        s_.stage_destroy()


def test_misuse_is_rejected_not_undefined(B):
    sc = SMALL["tiny"]
    inp, st, hz = _build(B, sc, with_successor=False)
    hz.begin_iteration()
    E = B.BambooError
    with pytest.raises(E) as e:
        st.stage_fwd(sc.M, hz.x[0], hz.y[0])
    assert e.value.status == B.E_BADMB
    with pytest.raises(E) as e:
        st.stage_bwd(0, hz.gz[0], hz.gx[0])                  # no stashed forward
    assert e.value.status == B.E_BADMB
    with pytest.raises(E) as e:
        st.shadow_fwd_frc(0, hz.y[0], hz.z_frc[0])           # forward not issued yet
    assert e.value.status == B.E_BADMB
    with pytest.raises(E) as e:
        st.shadow_bwd_brc(0, hz.gz[0], None)                 # BRC before any failover
    assert e.value.status == B.E_STATE
    st.stage_fwd(0, hz.x[0], hz.y[0])
    st.stage_fwd(1, hz.x[1], hz.y[1])
    with pytest.raises(E) as e:
        st.stage_fwd(2, hz.x[2], hz.y[2])                    # slot 0 still live (c_own = 2)
    assert e.value.status == B.E_BADMB
    st.shadow_fwd_frc(0, hz.y[0], None)                      # z may be NULL
    with pytest.raises(E) as e:
        st.shadow_fwd_frc(0, hz.y[0], None)
    assert e.value.status == B.E_BADMB
    # the size-query form of the schedule calls must not merge the stage: refused, the stage stays as it was
    before = st.stage_schedule()
    assert B.lib.failover_merge(st._h, 1, None, 0) == B.E_ARG
    small = (B.Instr * 2)()
    assert B.lib.failover_merge(st._h, 1, small, 2) == B.E_ARG
    assert st.stage_schedule() == before
    with pytest.raises(E) as e:
        st.shadow_bwd_brc(0, hz.gz[0], None)                 # still not merged
    assert e.value.status == B.E_STATE
    st.failover_merge(1)
    with pytest.raises(E) as e:
        st.failover_merge(1)
    assert e.value.status == B.E_STATE
    with pytest.raises(E) as e:
        st.shadow_bwd_brc(1, hz.gz[1], None)                 # slot never written
    assert e.value.status == B.E_STATE
    st.shadow_bwd_brc(0, hz.gz[0], None)
    st.stage_sync()
    st.stage_destroy()
    # no replica layers: every shadow call is refused
    sc0 = sc.replace(n_shadow=0)
    st2 = B.Stage(B.make_cfg(sc0), B.to_device(inp["own_w"].reshape(-1), sc.dtype), None)
    st2.stage_fwd(0, hz.x[0], hz.y[0])
    with pytest.raises(E) as e:
        st2.shadow_fwd_frc(0, hz.y[0], None)
    assert e.value.status == B.E_STATE
    st2.stage_sync()
    st2.stage_destroy()


def test_bubble_kernel_waits_about_as_long_as_asked(B):
    sc = SMALL["tiny"]
    inp, st, hz = _build(B, sc, with_successor=False)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    st.stage_bubble(1, 10.0)
    st.stage_sync()
    with torch.cuda.stream(st.stream_main):
        e0.record()
        st.stage_bubble(20, 100.0)          # 2 ms
        e1.record()
    st.stage_sync()
    ms = e0.elapsed_time(e1)
    assert 1.9 <= ms <= 3.0, ms
    st.stage_destroy()


@pytest.mark.parametrize("name,k_fail", [("tiny", 2), ("bf16_post_ln", 3), ("bf16_causal_d128", 0)])
@pytest.mark.parametrize("rc", ["LFLB", "EFEB"])
def test_rc_variants_recover_the_failure_free_gradients(B, name, k_fail, rc):
    """The lazy-FRC and eager-BRC variants of the paper's microbenchmarks (Section 7.4): same
    programs as the oracle's, and after a preemption the same gradients as the failure-free run of
    Bamboo's own variant, bitwise."""
    from paper_2204_12013_amd.harness import StageHarness, split_at_failure
    sc = SMALL[name]
    mode = {"LFLB": (B.RC_LFLB, S.LFLB), "EFEB": (B.RC_EFEB, S.EFEB)}[rc]
    inp, st0, hz0 = _build(B, sc)                       # reference: EFLB, no failure
    hz0.begin_iteration()
    hz0.run(st0.stage_schedule())
    hz0.sync()

    def build():
        st = B.Stage(B.make_cfg(sc, rc_mode=mode[0]), B.to_device(inp["own_w"].reshape(-1), sc.dtype),
                     B.to_device(inp["shadow_w"].reshape(-1), sc.dtype))
        scs = sc.replace(n_own=sc.n_shadow, n_shadow=0, stage_id=sc.stage_id + 1)
        succ = B.Stage(B.make_cfg(scs, frc_enabled=False), B.to_device(inp["shadow_w"].reshape(-1), sc.dtype), None)
        x = [B.to_device(inp["x"][k], sc.dtype) for k in range(sc.M)]
        gz = [B.to_device(inp["gz"][k], sc.dtype) for k in range(sc.M)]
        torch.cuda.synchronize()
        return st, StageHarness(st, x, gz, successor=succ)
    # failure-free iteration of the variant
    st1, hz1 = build()
    prog = st1.stage_schedule()
    assert prog == S.stage_program(sc.P, sc.stage_id, sc.M, rc=mode[1])
    hz1.begin_iteration()
    hz1.run(prog)
    hz1.sync()
    assert torch.equal(st1.own_g, st0.own_g)
    if rc == "EFEB":                                    # eager BRC reproduces the successor's gradients
        assert torch.equal(st1.shadow_g, hz0.succ.own_g)
    else:
        assert float(st1.shadow_g.abs().max()) == 0.0
    # the variant with the successor lost at k_fail
    st2, hz2 = build()
    hz2.begin_iteration()
    hz2.run(split_at_failure(prog, k_fail))
    hz2.succ.stage_sync()
    hz2.succ.own_g.zero_()
    merged = st2.failover_merge(k_fail)
    assert merged == S.failover_program(sc.P, sc.stage_id, sc.M, k_fail, rc=mode[1])
    hz2.run(merged)
    hz2.sync()
    assert torch.equal(st2.own_g, st0.own_g)
    assert torch.equal(st2.shadow_g, hz0.succ.own_g)
    for k in range(sc.M):
        assert torch.equal(hz2.gx[k], hz0.gx[k])
        assert torch.equal(hz2.z_frc[k], hz0.z_succ[k])
    # the iteration after the failover is the same merged program whatever ran eagerly before
    hz2.begin_iteration()
    assert st2.stage_schedule() == S.merged_program(sc.P, sc.stage_id, sc.M)
    hz2.run(st2.stage_schedule())
    hz2.sync()
    assert torch.equal(st2.own_g, st0.own_g) and torch.equal(st2.shadow_g, hz0.succ.own_g)
    for k in range(sc.M):
        assert torch.equal(hz2.gx[k], hz0.gx[k]) and torch.equal(hz2.z_frc[k], hz0.z_succ[k])
    for s_ in (st0, hz0.succ, st1, hz1.succ, st2, hz2.succ):
        s_.stage_destroy()


#                              name  arch dtype H heads  F  seq B own shadow P s M seed
DEGENERATE = {
    # one micro-batch, two stages: the program has a single forward and backward
    "one_microbatch": synth.StageConfig("d0", 0, 0, 64, 2, 128, 8, 2, 1, 1, 2, 0, 1, 41),
    # sequence length 1: every softmax is over one key; 3 tokens in all (the MFMA kernels do not cover it)
    "one_position_bf16": synth.StageConfig("d1", 1, 1, 64, 1, 128, 1, 3, 1, 1, 3, 1, 2, 42),
    # one head as wide as the model, one sample
    "one_head_one_sample": synth.StageConfig("d2", 1, 1, 128, 1, 256, 72, 1, 1, 1, 4, 2, 3, 43),
    # more replica layers than own layers (uneven partition), deep pipeline, few micro-batches
    "uneven_layers": synth.StageConfig("d3", 0, 1, 128, 2, 256, 40, 2, 1, 3, 6, 1, 2, 44),
}


@pytest.mark.parametrize("name", list(DEGENERATE))
def test_degenerate_configurations_match_oracle_with_and_without_failure(B, name):
    from paper_2204_12013_amd.harness import split_at_failure
    sc = DEGENERATE[name]
    tol = TOL[sc.dtype]
    inp, st, hz = _build(B, sc)
    prog = st.stage_schedule()
    assert prog == S.stage_program(sc.P, sc.stage_id, sc.M)
    hz.begin_iteration()
    hz.run(prog)
    hz.sync()
    ref = _oracle(sc, inp)
    for k in range(sc.M):
        assert_close(B.to_host(hz.y[k]), ref.y[k], tol, "stage B.to_host(hz.y[k])")
        assert_close(B.to_host(hz.gx[k]), ref.gx[k], tol, "stage B.to_host(hz.gx[k])")
        assert torch.equal(hz.z_frc[k], hz.z_succ[k])
    check_grads(st.own_g.cpu().numpy(), ref.G_own, sc.hidden, sc.ffn, tol, "own")
    check_grads(hz.succ.own_g.cpu().numpy(), ref.G_succ, sc.hidden, sc.ffn, tol, "successor")
    k_fail = sc.M - 1
    _, st2, hz2 = _build(B, sc)
    hz2.begin_iteration()
    hz2.run(split_at_failure(st2.stage_schedule(), k_fail))
    hz2.succ.stage_sync()
    hz2.succ.own_g.zero_()
    merged = st2.failover_merge(k_fail)
    assert merged == S.failover_program(sc.P, sc.stage_id, sc.M, k_fail)
    hz2.run(merged)
    hz2.sync()
    assert torch.equal(st2.own_g, st.own_g)
    assert torch.equal(st2.shadow_g, hz.succ.own_g)
    for s_ in (st, st2, hz.succ, hz2.succ):
        s_.stage_destroy()


def test_single_stage_pipeline_without_replica(B):
    """P = 1: no neighbours, no replica, no bubbles; only FNC and BNC remain."""
    from paper_2204_12013_amd.harness import StageHarness
    sc = synth.StageConfig("d4", 0, 1, 128, 2, 256, 24, 2, 2, 0, 1, 0, 3, 45)
    inp = synth.make_stage_inputs(sc)
    st = B.Stage(B.make_cfg(sc, frc_enabled=False), B.to_device(inp["own_w"].reshape(-1), sc.dtype), None)
    prog = st.stage_schedule()
    assert prog == S.stage_program(1, 0, sc.M, frc=False)
    assert not any(i[0] in (B.FRC, B.BRC, B.BUBBLE, B.SEND_ACT, B.RECV_GRAD) for i in prog)
    x = [B.to_device(inp["x"][k], sc.dtype) for k in range(sc.M)]
    gy = [B.to_device(inp["gz"][k], sc.dtype) for k in range(sc.M)]
    torch.cuda.synchronize()
    hz = StageHarness(st, x, gz=gy, gy_table=gy)
    hz.begin_iteration()
    hz.run(prog)
    hz.sync()
    own = oracle_layers(inp["own_w"], sc.hidden, sc.ffn)
    from oracle import layer as L
    G = None
    for k in range(sc.M):
        y, caches = L.stack_fwd(sc.arch, own, inp["x"][k].astype(np.float64), sc.micro_batch, sc.seq, sc.heads)
        gx, grads = L.stack_bwd(sc.arch, own, caches, inp["gz"][k].astype(np.float64))
        assert_close(B.to_host(hz.y[k]), y, TOL[sc.dtype], "stage B.to_host(hz.y[k])")
        assert_close(B.to_host(hz.gx[k]), gx, TOL[sc.dtype], "stage B.to_host(hz.gx[k])")
        G = grads if G is None else [{n: a[n] + b[n] for n in a} for a, b in zip(G, grads)]
    check_grads(st.own_g.cpu().numpy(), G, sc.hidden, sc.ffn, TOL[sc.dtype], "own")
    with pytest.raises(B.BambooError) as e:
        st.failover_merge(0)
    assert e.value.status == B.E_STATE
    st.stage_destroy()


@pytest.mark.parametrize("name", ["bf16_post_ln", "bf16_causal_d128"])
def test_gradients_do_not_depend_on_how_the_weight_gradients_are_launched(B, name):
    """With a token count the grouped weight-gradient launch covers (a multiple of 64), the four weight
    gradients of a layer and the ordered sums behind its bias / LayerNorm gradients go out as one launch;
    with a forced 64 x 64 tile every GEMM is launched singly and the sums get a launch of their own.  Both
    must match the oracle, and each other bitwise (the order of every sum is fixed by the data layout, not
    by the launch)."""
    sc = SMALL[name].replace(seq=128, micro_batch=2)
    assert (sc.micro_batch * sc.seq) % 64 == 0 and sc.micro_batch * sc.seq >= 192
    ref = None
    grads = []
    for tile in (0, 11):
        B.bk_gemm_tile(tile)
        try:
            inp, st, hz = _build(B, sc)
            hz.begin_iteration()
            hz.run(st.stage_schedule())
            hz.sync()
        finally:
            B.bk_gemm_tile(0)
        if ref is None:
            ref = _oracle(sc, inp)
        check_grads(st.own_g.cpu().numpy(), ref.G_own, sc.hidden, sc.ffn, TOL[sc.dtype], "own, tile %d" % tile)
        grads.append((st.own_g.clone(), hz.succ.own_g.clone(), [hz.gx[k].clone() for k in range(sc.M)]))
        st.stage_destroy()
        hz.succ.stage_destroy()
    assert torch.equal(grads[0][0], grads[1][0])
    assert torch.equal(grads[0][1], grads[1][1])
    for a, b in zip(grads[0][2], grads[1][2]):
        assert torch.equal(a, b)


@pytest.mark.parametrize("name,k_fail", [("tiny", 2), ("bf16_post_ln", 3), ("bf16_causal_d128", 0)])
def test_iteration_after_the_failover_runs_the_merged_program(B, name, k_fail):
    """Section 5.2: in the iterations after a preemption the shadow node executes all of the victim's
    instructions.  After failover_merge the next stage_begin_iteration installs the merged stage's
    whole-iteration program: it equals the oracle's list, the stage behaves as one stage of own + replica
    layers (against the oracle), and with the same parameters and inputs it ends with bitwise the
    gradients of the failure-free iteration (own, and the successor's in the replica buffer)."""
    from paper_2204_12013_amd.harness import split_at_failure
    sc = SMALL[name]
    tol = TOL[sc.dtype]
    inp, st0, hz0 = _build(B, sc)
    hz0.begin_iteration()
    hz0.run(st0.stage_schedule())
    hz0.sync()
    _, st, hz = _build(B, sc)
    hz.begin_iteration()
    hz.run(split_at_failure(st.stage_schedule(), k_fail))
    hz.succ.stage_sync()
    hz.run(st.failover_merge(k_fail))
    hz.sync()
    # second iteration: merged from the start
    hz.begin_iteration()
    prog = st.stage_schedule()
    assert prog == S.merged_program(sc.P, sc.stage_id, sc.M) == B.stage_merged_program(st.cfg)
    hz.run(prog)
    hz.sync()
    assert torch.equal(st.own_g, st0.own_g)
    assert torch.equal(st.shadow_g, hz0.succ.own_g)
    for k in range(sc.M):
        assert torch.equal(hz.gx[k], hz0.gx[k])
        assert torch.equal(hz.z_frc[k], hz0.z_succ[k])
        assert torch.equal(hz.gy[k], hz0.gy[k])            # BRC's input gradient is what the victim used to send
    own = oracle_layers(inp["own_w"], sc.hidden, sc.ffn)
    shadow = oracle_layers(inp["shadow_w"], sc.hidden, sc.ffn)
    x = {k: inp["x"][k].astype(np.float64) for k in range(sc.M)}
    gz = {k: inp["gz"][k].astype(np.float64) for k in range(sc.M)}
    sim = St.StageSim(sc.arch, own, shadow, sc.micro_batch, sc.seq, sc.heads, sc.P, sc.stage_id, sc.M, x, gz)
    sim.preempt_successor()
    sim.run(S.merged_program(sc.P, sc.stage_id, sc.M))
    check_grads(st.own_g.cpu().numpy(), sim.G_own, sc.hidden, sc.ffn, tol, "merged own")
    check_grads(st.shadow_g.cpu().numpy(), sim.G_shadow, sc.hidden, sc.ffn, tol, "merged replica")
    for k in range(sc.M):
        assert_close(B.to_host(hz.z_frc[k]), sim.z_frc[k], tol, "stage merged z")
        assert_close(B.to_host(hz.gx[k]), sim.gx[k], tol, "stage merged gx")
    for s_ in (st0, st, hz0.succ, hz.succ):
        s_.stage_destroy()


def test_stage_run_stops_where_the_hook_reports_a_lost_peer(B):
    """Section 4: a lost neighbour shows at a communication instruction.  stage_run hands every such
    instruction to the caller's hook and, when the hook says the peer is gone, stops before it and
    returns its index; the caller then merges and runs the failover schedule -- same gradients as a
    failure-free iteration, bitwise."""
    from paper_2204_12013_amd.harness import split_at_failure
    sc = SMALL["bf16_post_ln"]
    k_fail = 2
    inp, st0, hz0 = _build(B, sc)
    hz0.begin_iteration()
    hz0.run(st0.stage_schedule())
    hz0.sync()
    _, st, hz = _build(B, sc)
    hz.begin_iteration()
    prog = st.stage_schedule()
    seen = []

    def comm(op, lane, k, arg):
        seen.append((op, k))
        if op == B.SEND_ACT and k == k_fail and arg == sc.stage_id + 1:
            return True                                 # handing over micro-batch k_fail fails
        return hz._comm(op, lane, k, arg)
    n = st.stage_run(prog, x=hz.x, y=hz.y, z=hz.z_frc, gy=hz.gy, gx=hz.gx, gz=hz.gz, comm=comm)
    assert prog[n][0] == B.SEND_ACT and prog[n][2] == k_fail and 0 < n < len(prog)
    ran = prog[:n]
    assert ran[:len(split_at_failure(prog, k_fail))] == split_at_failure(prog, k_fail)      # FWD(k_fail) and its FRC ran
    assert all(i[0] in (B.BUBBLE, B.SEND_GRAD) for i in ran[len(split_at_failure(prog, k_fail)):])
    hz.bwd_done = {i[2] for i in prog[:n] if i[0] == B.BWD}
    hz.succ.stage_sync()
    hz.run(st.failover_merge(k_fail))
    hz.sync()
    assert torch.equal(st.own_g, st0.own_g) and torch.equal(st.shadow_g, hz0.succ.own_g)
    for k in range(sc.M):
        assert torch.equal(hz.gx[k], hz0.gx[k])
    # misuse: tables that an instruction needs are missing
    with pytest.raises(B.BambooError) as e:
        st.stage_begin_iteration()
        st.stage_run([(B.FWD, 0, 0, 0)], x=None, y=hz.y)
    assert e.value.status == B.E_ARG
    with pytest.raises(B.BambooError) as e:
        st.stage_run([(B.FWD, 0, sc.M, 0)], x=hz.x, y=hz.y)
    assert e.value.status == B.E_BADMB
    for s_ in (st0, st, hz0.succ, hz.succ):
        s_.stage_destroy()


@pytest.mark.parametrize("dtype,rc", [(0, 1), (1, 1), (1, 0)])
def test_pure_data_parallel_node_matches_oracle_and_recovers_the_peers_gradient(B, dtype, rc):
    """Section 5.2, "Support for Pure Data Parallelism": the node holds the whole model and the replica of a
    peer's model; eager FRC is the forward of the peer's minibatch beside its own (over-batching), lazy
    BRC rebuilds the peer's gradient when the peer is lost.  Against the oracle, and bitwise against a
    second stage object playing the peer."""
    from paper_2204_12013_amd.harness import StageHarness, split_at_failure
    sc = synth.StageConfig("dp", 1, dtype, 256 if dtype else 72, 4 if dtype else 3, 1024 if dtype else 200,
                           160 if dtype else 21, 2, 2, 2, 1, 0, 4, 31)
    tol = TOL[sc.dtype]
    inp = synth.make_stage_inputs(sc)
    peer_in = synth.make_stage_inputs(sc.replace(seed=sc.seed + 1))      # the peer's minibatch and upstream gradients
    dev = lambda a: B.to_device(a, sc.dtype)
    cfg = B.make_cfg(sc, rc_mode=rc, data_parallel=1)
    x, g = [dev(inp["x"][k]) for k in range(sc.M)], [dev(inp["gz"][k]) for k in range(sc.M)]
    xn, gn = [dev(peer_in["x"][k]) for k in range(sc.M)], [dev(peer_in["gz"][k]) for k in range(sc.M)]

    def node():
        st = B.Stage(cfg, dev(inp["own_w"].reshape(-1)), dev(inp["shadow_w"].reshape(-1)))
        return st, StageHarness(st, x, gn, gy_table=g, frc_in=xn)
    # the peer itself: its own model (= the replica's values) on its own minibatch
    peer = B.Stage(B.make_cfg(sc.replace(n_shadow=0), frc_enabled=False), dev(inp["shadow_w"].reshape(-1)), None)
    hp = StageHarness(peer, xn, gn, gy_table=gn)
    torch.cuda.synchronize()
    hp.begin_iteration()
    hp.run(peer.stage_schedule())
    hp.sync()
    st0, hz0 = node()
    prog = st0.stage_schedule()
    assert prog == S.stage_program(1, 0, sc.M, rc=rc)
    hz0.begin_iteration()
    hz0.run(prog)
    hz0.sync()
    if rc == 1:
        for k in range(sc.M):
            assert torch.equal(hz0.z_frc[k], hp.y[k])           # FRC == the peer's own forward, bitwise
    args = (sc.arch, oracle_layers(inp["own_w"], sc.hidden, sc.ffn), oracle_layers(inp["shadow_w"], sc.hidden, sc.ffn),
            sc.micro_batch, sc.seq, sc.heads, sc.M,
            {k: inp["x"][k].astype(np.float64) for k in range(sc.M)}, {k: inp["gz"][k].astype(np.float64) for k in range(sc.M)},
            {k: peer_in["x"][k].astype(np.float64) for k in range(sc.M)},
            {k: peer_in["gz"][k].astype(np.float64) for k in range(sc.M)})
    for k_fail in (0, 2, sc.M - 1):
        st, hz = node()
        hz.begin_iteration()
        hz.run(split_at_failure(prog, k_fail))
        merged = st.failover_merge(k_fail)
        assert merged == S.failover_program(1, 0, sc.M, k_fail, rc=rc, data_parallel=True)
        hz.run(merged)
        hz.sync()
        assert torch.equal(st.own_g, st0.own_g)
        assert torch.equal(st.shadow_g, peer.own_g)              # exactly what the peer would have contributed
        for k in range(sc.M):
            assert torch.equal(hz.gx[k], hz0.gx[k])
            assert torch.equal(hz.gy_replay[k], hp.gx[k])        # BRC's input gradient == the peer's own
        sim = St.DataParallelSim(*args)
        sim.run(S.prefix_until_failure(1, 0, sc.M, k_fail, rc=rc))
        sim.preempt_neighbour()
        sim.run(S.failover_program(1, 0, sc.M, k_fail, rc=rc, data_parallel=True))
        check_grads(st.own_g.cpu().numpy(), sim.G_own, sc.hidden, sc.ffn, tol, "data-parallel own")
        check_grads(st.shadow_g.cpu().numpy(), sim.G_shadow, sc.hidden, sc.ffn, tol, "data-parallel replica")
        for k in range(sc.M):
            assert_close(B.to_host(hz.z_frc[k]), sim.z_frc[k], tol, "stage data-parallel z")
            assert_close(B.to_host(hz.gx[k]), sim.gx[k], tol, "stage data-parallel gx")
        # the next iteration: both minibatches from the start
        hz.begin_iteration()
        assert st.stage_schedule() == S.merged_program(1, 0, sc.M)
        hz.run(st.stage_schedule())
        hz.sync()
        assert torch.equal(st.own_g, st0.own_g) and torch.equal(st.shadow_g, peer.own_g)
        st.stage_destroy()
    for s_ in (st0, peer):
        s_.stage_destroy()


def test_two_stages_driven_from_two_threads_give_the_results_of_sequential_runs(B):
    """The header allows one thread per stage, any number of stages per process: the launch state the library
    keeps per process (tile and ring choices, the activation table, the LDS size attributes of its kernels) must
    not care which thread gets there first.  Two different stages run three iterations each, concurrently, and
    must reproduce bitwise what each gives when it runs alone."""
    import threading
    names = ["bf16_post_ln", "bf16_causal_d128"]

    def run_one(name, out):
        try:
            sc = SMALL[name]
            inp, st, hz = _build(B, sc)
            prog = st.stage_schedule()
            for _ in range(3):
                hz.begin_iteration()
                hz.run(prog)
            hz.sync()
            torch.cuda.synchronize()
            out[name] = ([t.clone() for t in hz.y] + [t.clone() for t in hz.z_frc] + [t.clone() for t in hz.gx],
                         st.own_g.clone(), hz.succ.own_g.clone())
            st.stage_destroy()
            hz.succ.stage_destroy()
        except Exception as e:          # surfaces in the main thread below
            out[name] = e

    alone, together = {}, {}
    # the threads go first: in a fresh process they also race for the one-time set-up
    threads = [threading.Thread(target=run_one, args=(n, together)) for n in names]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
        assert not t.is_alive()
    for n in names:
        run_one(n, alone)
    for n in names:
        for res in (alone[n], together[n]):
            if isinstance(res, Exception):
                raise res
        (acts_a, g_a, gs_a), (acts_t, g_t, gs_t) = alone[n], together[n]
        assert all(torch.equal(a, b) for a, b in zip(acts_a, acts_t)), n
        assert torch.equal(g_a, g_t) and torch.equal(gs_a, gs_t), n
