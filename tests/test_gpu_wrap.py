"""The wrap-around stage through the C ABI (GPU only): the last stage with the LM head and loss,
shadowing the first stage with its embedding (Section 5.1).  Against the oracle at the stated
tolerance, and the paper's two invariants on the GPU itself, bitwise: FRC is the first stage's
forward, and a failover ends with the gradients of the failure-free run."""
import numpy as np
import pytest
import torch

from oracle import ends as E
from oracle import schedule as S
from oracle import stage as St
from paper_2204_12013_amd import synth
from util import TOL, assert_close, check_grads, oracle_layers, rel_l2

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

#                         name  arch dtype  H  heads  F   seq  B  own shadow P  s  M  seed      vocab
WRAP = {
    "fp32_encoder": (synth.StageConfig("w0", 0, 0, 64, 2, 256, 16, 2, 1, 1, 3, 2, 4, 31), 96),
    "fp32_decoder_two_stages": (synth.StageConfig("w1", 1, 0, 72, 3, 200, 21, 3, 1, 2, 2, 1, 3, 32), 104),
    "bf16_decoder": (synth.StageConfig("w2", 1, 1, 256, 2, 768, 160, 1, 2, 2, 4, 3, 4, 33), 1000),
    "bf16_encoder": (synth.StageConfig("w3", 0, 1, 256, 4, 1024, 200, 2, 2, 2, 4, 3, 5, 34), 2048),
}


@pytest.fixture(scope="module")
def B():
    from paper_2204_12013_amd import binding
    return binding


def _ids(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def _build(B, sc, V, swap_slots=0, rc_mode=None):
    from paper_2204_12013_amd.harness import WrapHarness
    inp = synth.make_stage_inputs(sc)
    ein = synth.make_ends_inputs(sc, V)
    cfg = B.make_cfg(sc, wrap=1, swap_slots=swap_slots, rc_mode=rc_mode)
    st = B.Stage(cfg, B.to_device(inp["own_w"].reshape(-1), sc.dtype), B.to_device(inp["shadow_w"].reshape(-1), sc.dtype))
    en = B.Ends(cfg, V, B.to_device(ein["front_w"], sc.dtype), B.to_device(ein["back_w"], sc.dtype))
    x = [B.to_device(inp["x"][k], sc.dtype) for k in range(sc.M)]
    g1 = [B.to_device(ein["g1"][k], sc.dtype) for k in range(sc.M)]
    ids = [_ids(ein["ids"][k]) for k in range(sc.M)]
    labels = [_ids(ein["labels"][k]) for k in range(sc.M)]
    torch.cuda.synchronize()
    return inp, ein, st, en, WrapHarness(st, en, x, ids, labels, g1)


def _first_stage(B, sc, V, inp, ein):
    """The first stage itself: its layers are the replica's, its front end the same embedding.  Runs
    forward and backward of every micro-batch; returns (outputs, layer gradients, front gradients)."""
    sc0 = sc.replace(n_own=sc.n_shadow, n_shadow=0, stage_id=0)
    cfg0 = B.make_cfg(sc0, frc_enabled=False)
    st0 = B.Stage(cfg0, B.to_device(inp["shadow_w"].reshape(-1), sc.dtype), None)
    en0 = B.Ends(cfg0, V, B.to_device(ein["front_w"], sc.dtype), B.to_device(ein["back_w"], sc.dtype))
    st0.stage_begin_iteration()
    st0.zero_grads()
    zs, keep = [], []
    main = st0.stream_main
    ids = [_ids(ein["ids"][k]) for k in range(sc.M)]
    g1 = [B.to_device(ein["g1"][k], sc.dtype) for k in range(sc.M)]
    torch.cuda.synchronize()
    for k in range(sc.M):                       # one at a time: slot discipline of stage 0 does not matter here
        x0, z, dx0 = st0.new_act(), st0.new_act(), st0.new_act()
        en0.ends_front_fwd(k, ids[k], x0, main)
        st0.stage_fwd(k, x0, z)
        st0.stage_bwd(k, g1[k], dx0)
        en0.ends_front_bwd(k, dx0, main)
        zs.append(z)
        keep += [x0, dx0]                       # buffers stay alive until the work on them has run
    st0.stage_sync()
    out = zs, st0.own_g.clone(), en0.front_g.clone()
    st0.stage_destroy()
    en0.ends_destroy()
    return out


def _oracle(sc, V, inp, ein, k_fail=None):
    own = oracle_layers(inp["own_w"], sc.hidden, sc.ffn)
    shadow = oracle_layers(inp["shadow_w"], sc.hidden, sc.ffn)
    front = E.unpack_front(ein["front_w"], sc.arch, V, sc.seq, sc.hidden)
    back = E.unpack_back(ein["back_w"], sc.arch, V, sc.hidden)
    x = {k: inp["x"][k].astype(np.float64) for k in range(sc.M)}
    g1 = {k: ein["g1"][k].astype(np.float64) for k in range(sc.M)}
    ids = {k: ein["ids"][k].astype(np.int64) for k in range(sc.M)}
    labels = {k: ein["labels"][k].astype(np.int64) for k in range(sc.M)}
    sim = St.WrapStageSim(sc.arch, own, back, shadow, front, sc.micro_batch, sc.seq, sc.heads, sc.P, sc.M,
                          x, labels, ids, g1)
    if k_fail is None:
        return sim.run(S.stage_program(sc.P, sc.P - 1, sc.M))
    sim.run(S.prefix_until_failure(sc.P, sc.P - 1, sc.M, k_fail))
    return sim.run(S.wrap_failover_program(sc.P, sc.M, k_fail))


def _check_named(got_flat, want, unpack, tol, label):
    got = unpack(got_flat.cpu().numpy())
    for n, w in want.items():
        assert_close(got[n], w, tol, "wrap %s gradient: %s" % (label, n))


def _check_against_oracle(B, sc, V, st, en, hz, ref):
    tol = TOL[sc.dtype]
    check_grads(st.own_g.cpu().numpy(), ref.G_own, sc.hidden, sc.ffn, tol, "own")
    _check_named(en.back_g, ref.G_back, lambda a: E.unpack_back(a, sc.arch, V, sc.hidden), tol, "back")
    loss = hz.loss.cpu().numpy()
    for k in range(sc.M):
        assert abs(loss[k] - ref.loss[k]) <= tol * abs(ref.loss[k]), (k, loss[k], ref.loss[k])
        assert_close(B.to_host(hz.gx[k]), ref.gx[k], tol, "wrap B.to_host(hz.gx[k])")
        assert_close(B.to_host(hz.z_frc[k]), ref.z_frc[k], tol, "wrap B.to_host(hz.z_frc[k])")


@pytest.mark.parametrize("name", list(WRAP))
def test_iteration_matches_oracle_and_frc_is_the_first_stage_forward(B, name):
    sc, V = WRAP[name]
    inp, ein, st, en, hz = _build(B, sc, V)
    prog = st.stage_schedule()
    assert prog == S.stage_program(sc.P, sc.P - 1, sc.M)
    hz.begin_iteration()
    hz.run(prog)
    hz.sync()
    ref = _oracle(sc, V, inp, ein)
    _check_against_oracle(B, sc, V, st, en, hz, ref)
    assert float(st.shadow_g.abs().max()) == 0.0 and float(en.front_g.abs().max()) == 0.0    # BRC is lazy
    zs, _, _ = _first_stage(B, sc, V, inp, ein)
    for k in range(sc.M):
        assert torch.equal(hz.z_frc[k], zs[k])
    # a second iteration gives the same bits
    own_g, back_g, loss = st.own_g.clone(), en.back_g.clone(), hz.loss.clone()
    hz.begin_iteration()
    hz.run(prog)
    hz.sync()
    assert torch.equal(st.own_g, own_g) and torch.equal(en.back_g, back_g) and torch.equal(hz.loss, loss)
    st.stage_destroy()
    en.ends_destroy()


@pytest.mark.parametrize("name,k_fail", [("fp32_encoder", 0), ("fp32_encoder", 3), ("fp32_decoder_two_stages", 1),
                                         ("fp32_decoder_two_stages", 2), ("bf16_decoder", 2), ("bf16_encoder", 1),
                                         ("bf16_encoder", 4)])
def test_failover_rebuilds_the_first_stage_gradients(B, name, k_fail):
    from paper_2204_12013_amd.harness import split_at_failure
    sc, V = WRAP[name]
    inp, ein, st0, en0, hz0 = _build(B, sc, V)            # failure-free run
    hz0.begin_iteration()
    hz0.run(st0.stage_schedule())
    hz0.sync()
    zs, first_g, first_front_g = _first_stage(B, sc, V, inp, ein)
    _, _, st, en, hz = _build(B, sc, V)
    hz.begin_iteration()
    hz.run(split_at_failure(st.stage_schedule(), k_fail))
    merged = st.failover_merge(k_fail)
    assert merged == S.wrap_failover_program(sc.P, sc.M, k_fail)
    assert st.stage_schedule() == merged
    hz.run(merged)
    hz.sync()
    ref = _oracle(sc, V, inp, ein, k_fail)
    _check_against_oracle(B, sc, V, st, en, hz, ref)
    tol = TOL[sc.dtype]
    check_grads(st.shadow_g.cpu().numpy(), ref.G_shadow, sc.hidden, sc.ffn, tol, "replica")
    _check_named(en.front_g, ref.G_front, lambda a: E.unpack_front(a, sc.arch, V, sc.seq, sc.hidden), tol, "front")
    # nothing is lost: the own side equals the failure-free run, the replica side what the victim would hold
    assert torch.equal(st.own_g, st0.own_g) and torch.equal(en.back_g, en0.back_g)
    assert torch.equal(hz.loss, hz0.loss)
    assert torch.equal(st.shadow_g, first_g) and torch.equal(en.front_g, first_front_g)
    for k in range(sc.M):
        assert torch.equal(hz.gx[k], hz0.gx[k])
        assert torch.equal(hz.z_frc[k], zs[k])
    for o in (st0, st):
        o.stage_destroy()
    for o in (en0, en):
        o.ends_destroy()


@pytest.mark.parametrize("name,k_fail,slots", [("fp32_encoder", 1, 1), ("bf16_decoder", 2, 2), ("bf16_encoder", 3, 2)])
def test_wrap_around_with_swap_out_of_the_replica_stash(B, name, k_fail, slots):
    """The replica layers' FRC results swapped out to the host (the front end's small stash stays on the
    device): failover gives bitwise the gradients of the device-resident failure-free run."""
    from paper_2204_12013_amd.harness import split_at_failure
    sc, V = WRAP[name]
    inp, ein, st0, en0, hz0 = _build(B, sc, V)
    hz0.begin_iteration()
    hz0.run(st0.stage_schedule())
    hz0.sync()
    _, first_g, first_front_g = _first_stage(B, sc, V, inp, ein)
    _, _, st, en, hz = _build(B, sc, V, swap_slots=slots)
    hz.begin_iteration()
    hz.run(split_at_failure(st.stage_schedule(), k_fail))
    hz.run(st.failover_merge(k_fail))
    hz.sync()
    assert torch.equal(st.own_g, st0.own_g) and torch.equal(en.back_g, en0.back_g) and torch.equal(hz.loss, hz0.loss)
    assert torch.equal(st.shadow_g, first_g) and torch.equal(en.front_g, first_front_g)
    for o in (st0, st):
        o.stage_destroy()
    for o in (en0, en):
        o.ends_destroy()


def test_wrap_misuse_is_rejected(B):
    sc, V = WRAP["fp32_encoder"]
    inp, ein, st, en, hz = _build(B, sc, V)
    hz.begin_iteration()
    with pytest.raises(B.BambooError) as e:                 # no forward yet
        en.ends_back_bwd(hz.gy[0], st.stream_main)
    assert e.value.status == B.E_STATE
    with pytest.raises(B.BambooError) as e:
        en.ends_front_bwd(1, hz.dx0[1], st.stream_main)
    assert e.value.status == B.E_BADMB
    with pytest.raises(B.BambooError) as e:
        en.ends_front_fwd(sc.M, hz.ids[0], hz.x0[0], st.stream_main)
    assert e.value.status == B.E_BADMB
    # FRC of a wrap-around stage does not need this stage's forward of the micro-batch
    en.ends_front_fwd(2, hz.ids[2], hz.x0[2], st.stream_frc)
    st.shadow_fwd_frc(2, hz.x0[2], hz.z_frc[2])
    st.stage_sync()
    st.stage_destroy()
    en.ends_destroy()


def test_ends_at_the_bert_large_size(B):
    """The model's ends at the size bench.py times them (4096 tokens, hidden 1024, vocabulary 30528,
    Zipf-distributed ids): loss, head gradients, input gradient and embedding gradients against the oracle."""
    sc = synth.CONFIGS["bert_large_stage"].replace(stage_id=3, M=1)
    V = synth.VOCAB["bert_large_stage"]
    cfg = B.make_cfg(sc, wrap=1)
    ein = synth.make_ends_inputs(sc, V)
    rng = np.random.default_rng(9)
    y = synth.round_to_storage(rng.standard_normal((sc.tokens, sc.hidden), dtype=np.float32), sc.dtype)
    dx0 = synth.round_to_storage(rng.standard_normal((sc.tokens, sc.hidden), dtype=np.float32) / 64, sc.dtype)
    en = B.Ends(cfg, V, B.to_device(ein["front_w"], sc.dtype), B.to_device(ein["back_w"], sc.dtype))
    s = torch.cuda.current_stream()
    d_y, d_dx0 = B.to_device(y, sc.dtype), B.to_device(dx0, sc.dtype)
    ids, labels = _ids(ein["ids"][0]), _ids(ein["labels"][0])
    loss = torch.zeros(1, dtype=torch.float32, device=DEV)
    gy = torch.empty_like(d_y)
    x0 = torch.empty_like(d_y)
    en.ends_begin_iteration()
    en.ends_back_fwd(d_y, labels, loss, s)
    en.ends_back_bwd(gy, s)
    en.ends_front_fwd(0, ids, x0, s)
    en.ends_front_bwd(0, d_dx0, s)
    torch.cuda.synchronize()
    tol = TOL[sc.dtype]
    back = E.unpack_back(ein["back_w"], sc.arch, V, sc.hidden)
    want_loss, _, cache = E.back_fwd(sc.arch, back, y.astype(np.float64), ein["labels"][0].astype(np.int64))
    want_gy, want_gb = E.back_bwd(sc.arch, back, cache)
    assert abs(loss.item() - want_loss) <= tol * want_loss
    assert_close(B.to_host(gy), want_gy, tol, "wrap B.to_host(gy)")
    _check_named(en.back_g, want_gb, lambda a: E.unpack_back(a, sc.arch, V, sc.hidden), tol, "back")
    del cache, want_gb
    front = E.unpack_front(ein["front_w"], sc.arch, V, sc.seq, sc.hidden)
    want_x0, cf = E.front_fwd(sc.arch, front, ein["ids"][0].astype(np.int64), sc.seq)
    assert_close(B.to_host(x0), want_x0, tol, "wrap B.to_host(x0)")
    want_gf = E.front_bwd(sc.arch, front, cf, dx0.astype(np.float64))
    _check_named(en.front_g, want_gf, lambda a: E.unpack_front(a, sc.arch, V, sc.seq, sc.hidden), tol, "front")
    en.ends_destroy()


@pytest.mark.parametrize("name,k_fail", [("fp32_encoder", 2), ("bf16_decoder", 1), ("bf16_encoder", 3)])
def test_lazy_frc_variant_and_the_iteration_after_the_failover(B, name, k_fail):
    """The wrap-around stage under the lazy variant of Section 7.4 (nothing redundant runs until the first stage
    is lost; the failover schedule then runs FRC before every BRC), and, for both variants, the iteration
    AFTER the failover, in which the last stage executes all of the first stage's instructions (Section 5.2):
    program equal to the oracle's, gradients bitwise those of the failure-free pair of stages."""
    from paper_2204_12013_amd.harness import split_at_failure
    sc, V = WRAP[name]
    inp, ein, st0, en0, hz0 = _build(B, sc, V)            # failure-free run, eager FRC
    hz0.begin_iteration()
    hz0.run(st0.stage_schedule())
    hz0.sync()
    zs, first_g, first_front_g = _first_stage(B, sc, V, inp, ein)
    _, _, st, en, hz = _build(B, sc, V, rc_mode=B.RC_LFLB)
    prog = st.stage_schedule()
    assert prog == S.stage_program(sc.P, sc.P - 1, sc.M, rc=S.LFLB) and not any(i[0] == B.FRC for i in prog)
    hz.begin_iteration()
    hz.run(split_at_failure(prog, k_fail))
    merged = st.failover_merge(k_fail)
    assert merged == S.wrap_failover_program(sc.P, sc.M, k_fail, rc=S.LFLB)
    hz.run(merged)
    hz.sync()

    def same_as_failure_free():
        assert torch.equal(st.own_g, st0.own_g) and torch.equal(en.back_g, en0.back_g)
        assert torch.equal(hz.loss, hz0.loss)
        assert torch.equal(st.shadow_g, first_g) and torch.equal(en.front_g, first_front_g)
        for k in range(sc.M):
            assert torch.equal(hz.gx[k], hz0.gx[k])
            assert torch.equal(hz.z_frc[k], zs[k])
    same_as_failure_free()
    # the next iteration: the whole-iteration program of the merged ends of the pipeline
    hz.begin_iteration()
    prog2 = st.stage_schedule()
    assert prog2 == S.wrap_merged_program(sc.P, sc.M) == B.stage_merged_program(st.cfg)
    hz.run(prog2)
    hz.sync()
    same_as_failure_free()
    for o in (st0, st):
        o.stage_destroy()
    for o in (en0, en):
        o.ends_destroy()
