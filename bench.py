#!/usr/bin/env python3
"""Benchmark of the Bamboo stage hot path on one MI355X.

A step is one training iteration of the stage: the stage's instruction list for
all M micro-batches (forward + backward over the own layers, eager FRC over the
replica layers on the second lane).  Inputs are synthetic, seeded, and resident
in HBM before the timed region.  Prints one JSON line.

Modes (all reported; `value` is mode B):
  A  FRC off, no bubbles      pure stage compute
  B  FRC on,  no bubbles      FRC fully exposed (worst case)
  C  FRC off / on with the simulated 1F1B bubbles of the slot timeline
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK = {"mfma_bf16": 2.5e15, "hbm": 8.0e12, "fp32_vector": 157.3e12}


def _iteration_flops(sc, frc):
    T, H, S, F = sc.tokens, sc.hidden, sc.seq, sc.ffn
    gemm_fwd = 2.0 * T * (3 * H * H + H * H + 2 * H * F)
    attn_fwd = 4.0 * T * S * H * (0.5 if sc.arch == 1 else 1.0)
    fwd = gemm_fwd + attn_fwd
    bwd = 2.0 * gemm_fwd + 2.5 * attn_fwd
    return sc.M * (sc.n_own * (fwd + bwd) + (sc.n_shadow * fwd if frc else 0.0))


def _replay_end(B, merged):
    """Index where the failover schedule stops rebuilding lost state and resumes the merged 1F1B
    groups: the first send of an FRC output to the stage after the victim, or, where there is no
    such stage, the BRC that belongs to the first backward group."""
    for i, ins in enumerate(merged):
        if ins[0] == B.SEND_ACT:
            return i
        if ins[0] in (B.BWD, B.FWD):
            while i > 0 and merged[i - 1][0] in (B.BRC, B.RECV_GRAD, B.RECV_ACT, B.SEND_GRAD):
                i -= 1
                if merged[i][0] == B.BRC:
                    break
            return i
    return len(merged)


def _profiled_traffic(workload, site):
    """HBM bytes per launch of one launch site (or of the average stage-GEMM launch, site "stage_gemm") from
    the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter
    reads for the library's copy kernel of known size), or None where no summary covers it."""
    path = os.path.join(ROOT, "profiles", "%s_pmc_traffic.txt" % workload)
    try:
        for line in open(path):
            if line.startswith("%s_traffic_bytes_per_launch=" % site):
                return int(line.split("=")[1])
    except OSError:
        pass
    return None


def _cpu_baseline(sc, seconds_budget=12.0, flop_rate_guess=2.0e11):
    """The oracle as it stands (numpy/BLAS fp64), timed on the host: layers of this workload forward + backward
    on one micro-batch -- as many layer passes as fit the time budget, at least one, at most four times the
    stage's layer count --, extrapolated linearly to an iteration (flops are linear in layers x micro-batches).
    Where one layer pass at the full sequence length would blow the budget (the large-layer stage: 4.5e13 flop),
    the sample is a micro-batch of the same layer at a shorter sequence, scaled by the token count."""
    import numpy as np
    from oracle import layer as L
    from paper_2204_12013_amd import synth
    seq = sc.seq
    while seq > 64 and 72.0 * sc.micro_batch * seq * sc.hidden ** 2 > seconds_budget * flop_rate_guess:
        seq //= 2
    one = sc.replace(n_own=1, n_shadow=0, seq=seq)
    inp = synth.make_stage_inputs(one, n_microbatches=1)
    p = L.unpack_layer(inp["own_w"][0].astype(np.float64), sc.hidden, sc.ffn)
    x = inp["x"][0].astype(np.float64)
    g = inp["gz"][0].astype(np.float64)
    t_f = t_b = 0.0
    n = 0
    # layers beyond the stage's own count are further samples of the same measurement (same shapes)
    while n < 4 * sc.n_own and (n == 0 or (t_f + t_b) * (n + 1) / n <= seconds_budget):
        t0 = time.perf_counter()
        x, cache = L.layer_fwd(sc.arch, p, x, one.micro_batch, one.seq, sc.heads)
        t1 = time.perf_counter()
        g, _ = L.layer_bwd(sc.arch, p, cache, g)
        t2 = time.perf_counter()
        t_f, t_b, n = t_f + (t1 - t0), t_b + (t2 - t1), n + 1
    scale = sc.seq / seq
    t_iter = sc.M * (sc.n_own * (t_f + t_b) + sc.n_shadow * t_f) / n * scale
    try:
        import threadpoolctl
        cores = max([i.get("num_threads", 1) for i in threadpoolctl.threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": sc.M * sc.micro_batch / t_iter, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "sample": "fp64 oracle (numpy, matrix products through BLAS), %d layer(s) forward (%.2f s) + backward "
                      "(%.2f s) on 1 micro-batch of %s%s, extrapolated to the FRC-on iteration (%d micro-batches x "
                      "(%d own fwd+bwd + %d replica fwd))"
                      % (n, t_f, t_b, sc.name,
                         "" if seq == sc.seq else " cut to sequence length %d (times scaled by %d tokens / %d)"
                         % (seq, sc.tokens, one.tokens), sc.M, sc.n_own, sc.n_shadow)}


GEMM_SITES = ("gemm_qkv", "gemm_attn_out", "gemm_ffn1", "gemm_ffn2", "dgrad_ffn2", "dgrad_ffn1", "dgrad_attn_out",
              "dgrad_qkv", "wgrad_group")
SITE_KERNEL = {   # what each timed site launches
    "gemm_qkv": "gemm_mfma_pl_kernel, forward form with bias (QKV projection)",
    "gemm_attn_out": "gemm_mfma_pl_kernel, forward form with bias + residual (attention output projection)",
    "gemm_ffn1": "gemm_mfma_pl_kernel, forward form with bias + GELU and its derivative (first FFN GEMM)",
    "gemm_ffn2": "gemm_mfma_pl_kernel, forward form with bias + residual (second FFN GEMM)",
    "dgrad_ffn2": "gemm_mfma_pl_kernel, input-gradient form times the stored GELU derivative, with column sums",
    "dgrad_ffn1": "gemm_mfma_pl_kernel, input-gradient form (through the first FFN GEMM)",
    "dgrad_attn_out": "gemm_mfma_pl_kernel, input-gradient form (through the attention output projection)",
    "dgrad_qkv": "gemm_mfma_pl_kernel, input-gradient form (through the QKV projection)",
    "wgrad_group": "gemm_mfma_pl_group_kernel: the four weight gradients of a layer in one launch, fp32 accumulate",
}


def _make_inputs(torch, synth, sc, dev):
    """Parameters and per-micro-batch tensors of the workload's distributions, drawn on the device."""
    act = torch.bfloat16 if sc.dtype == 1 else torch.float32
    gen = torch.Generator(device=dev)
    gen.manual_seed(sc.seed)

    def layer_stack(n):
        H, F = sc.hidden, sc.ffn
        out = []
        for _ in range(n):
            for name in synth.PARAM_NAMES:
                numel = 1
                for s_ in synth.param_shapes(H, F)[name]:
                    numel *= s_
                v = torch.randn(numel, generator=gen, device=dev, dtype=torch.float32) * 0.02
                if name in ("g1", "g2"):
                    v += 1.0
                out.append(v.to(act))
                del v
        return torch.cat(out)
    T, H, M = sc.tokens, sc.hidden, sc.M
    own, shadow = layer_stack(sc.n_own), layer_stack(sc.n_shadow)
    x = [torch.randn(T, H, generator=gen, device=dev, dtype=torch.float32).to(act) for _ in range(M)]
    gy = [(torch.randn(T, H, generator=gen, device=dev, dtype=torch.float32) / (T * H) ** 0.5).to(act)
          for _ in range(M)]
    return gen, act, own, shadow, x, gy


def _time_iters(torch, hz, prog, n, us_per_tick=0.0):
    """n iterations of the instruction list, bracketed by device synchronisation; ms per iteration."""
    hz.us_per_tick = us_per_tick
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(n):
        hz.begin_iteration(zero_grads=True)
        hz.run(prog)
    hz.sync()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / max(n, 1)


def _site_profile(B, st, torch, hz, prog, k_p):
    """The iteration again with an event pair around every launch, on the launch's own stream."""
    st.stage_profile(True)
    _time_iters(torch, hz, prog, k_p)
    sites = {}
    for i, name in enumerate(B.KERNEL_CLASSES):
        ms, n, work = st.stage_profile_read(i)
        if n:
            sites[name] = {"launches": n, "avg_us": ms * 1e3 / n, "ms_per_step": ms / k_p, "rate": work / (ms * 1e-3),
                           "work_per_launch": work / n}
    st.stage_profile(False)
    return sites


def _roofline(sc, sites, k_p, two_lanes):
    """`roofline` of one workload: the single launch site with the most time per iteration (the dominant
    kernel), measured live (algorithmic flops per launch / average launch duration), beside the aggregate
    over all stage GEMM launches, which is what the 60 % target is stated on."""
    gemm = {k: v for k, v in sites.items() if k in GEMM_SITES}
    dom = max(gemm, key=lambda k: gemm[k]["ms_per_step"])
    d = gemm[dom]
    g_ms = sum(v["avg_us"] * v["launches"] for v in gemm.values()) * 1e-3
    g_work = sum(v["work_per_launch"] * v["launches"] for v in gemm.values())
    g_n = sum(v["launches"] for v in gemm.values())
    agg = g_work / (g_ms * 1e-3)
    measured = ("HIP event pair around every launch of %d iteration(s), %s"
                % (k_p, "FRC on (two lanes)" if two_lanes else "FRC off (one lane, no contention between lanes)"))
    return {"kernel": SITE_KERNEL[dom], "site": dom, "bound": "mfma", "achieved": d["rate"] / 1e12,
            "peak": PEAK["mfma_bf16"] / 1e12, "unit": "TFLOP/s", "frac": d["rate"] / PEAK["mfma_bf16"],
            "traffic": _profiled_traffic(sc.name, dom), "avg_launch_us": d["avg_us"],
            "flops_per_launch": d["work_per_launch"], "launches_per_step": d["launches"] // k_p,
            "share_of_gemm_time": d["ms_per_step"] * k_p / g_ms,
            "stage_gemms": {"achieved": agg / 1e12, "frac": agg / PEAK["mfma_bf16"], "launches_per_step": g_n // k_p,
                            "avg_launch_us": g_ms * 1e3 / g_n, "flops_per_launch": g_work / g_n,
                            "traffic": _profiled_traffic(sc.name, "stage_gemm")},
            "measured": measured}


def _kernel_table(sites, k_p):
    flop_sites = GEMM_SITES + ("attn_fwd", "attn_bwd")
    out = {}
    for k, v in sites.items():
        unit = "TFLOP/s" if k in flop_sites else "GB/s"
        rate = v["rate"] / (1e12 if k in flop_sites else 1e9)
        out[k] = {"avg_us": v["avg_us"], "launches_per_step": v["launches"] // k_p, "ms_per_step": v["ms_per_step"],
                  unit: rate, "frac_of_peak": v["rate"] / (PEAK["mfma_bf16"] if k in flop_sites else PEAK["hbm"])}
    return out


def measure_core(B, synth, torch, sc, steps, warmup, two_lanes=False, cpu_baseline=True, roofline_only=False):
    """Modes A, B, C, the per-site timing and the roofline of one workload; returns (record, live objects)."""
    from paper_2204_12013_amd.harness import StageHarness
    dev = torch.device("cuda:0")
    gen, act, own, shadow, x, gy = _make_inputs(torch, synth, sc, dev)
    cfg = B.make_cfg(sc, frc_enabled=True)
    st = B.Stage(cfg, own, shadow)
    del own, shadow
    M = sc.M
    torch.cuda.synchronize()
    hz = StageHarness(st, x, gz=gy, gy_table=gy)
    prog_on = st.stage_schedule()
    prog_off = [i for i in prog_on if i[0] != B.FRC]
    if roofline_only:
        # profiler aid: nothing but warm-up and the per-site pass, so that a kernel trace of this run averages
        # exactly the launches the roofline block is computed from
        prog = prog_on if two_lanes else prog_off
        _time_iters(torch, hz, prog, warmup)
        sites = _site_profile(B, st, torch, hz, prog, steps)
        rec = {"config": {"workload": sc.name}, "roofline": _roofline(sc, sites, steps, two_lanes),
               "kernel_sites": _kernel_table(sites, steps)}
        return rec, {"st": st, "hz": hz, "x": x, "gy": gy}
    _time_iters(torch, hz, prog_on, warmup)
    ms_on = _time_iters(torch, hz, prog_on, steps)                       # mode B: the headline
    rec = {"value": M * sc.micro_batch / (ms_on * 1e-3), "unit": "samples/s", "steps": steps, "warmup": warmup,
           "ms_per_step": ms_on, "dtype": "bf16" if sc.dtype == 1 else "f32",
           "config": {"workload": sc.name, "arch": "post-LN encoder" if sc.arch == 0 else "pre-LN causal decoder",
                      "hidden": sc.hidden, "heads": sc.heads, "ffn": sc.ffn, "seq": sc.seq,
                      "micro_batch": sc.micro_batch, "micro_batches": M, "own_layers": sc.n_own,
                      "replica_layers": sc.n_shadow, "pipeline_depth": sc.P, "stage_id": sc.stage_id,
                      "mode": "B: FRC on, no simulated bubbles"}}
    rec["mfma_util_end_to_end"] = _iteration_flops(sc, True) / (ms_on * 1e-3) / PEAK["mfma_bf16"]
    _time_iters(torch, hz, prog_off, 1)
    ms_off = _time_iters(torch, hz, prog_off, steps)                     # mode A
    rec["samples_per_s_frc_off"] = M * sc.micro_batch / (ms_off * 1e-3)
    rec["ms_per_step_frc_off"] = ms_off
    rec["frc_overhead_pct_no_bubbles"] = 100.0 * (ms_on - ms_off) / ms_off
    # mode C: bubbles sized from the failure-free iteration (one tick = one forward)
    us_per_tick = ms_off * 1e3 / (M * (cfg.tick_F + cfg.tick_B))
    k_c = max(2, min(steps, 5))
    ms_c_off = _time_iters(torch, hz, prog_off, k_c, us_per_tick)
    ms_c_on = _time_iters(torch, hz, prog_on, k_c, us_per_tick)
    rec["bubble_mode"] = {"us_per_tick": us_per_tick, "ms_per_step_frc_off": ms_c_off, "ms_per_step_frc_on": ms_c_on,
                          "frc_overhead_pct": 100.0 * (ms_c_on - ms_c_off) / ms_c_off, "steps": k_c}
    if sc.dtype == 1:
        k_p = max(1, min(steps, 3))
        sites = _site_profile(B, st, torch, hz, prog_on if two_lanes else prog_off, k_p)
        rec["roofline"] = _roofline(sc, sites, k_p, two_lanes)
        rec["mfma_util_stage_gemms"] = rec["roofline"]["stage_gemms"]["frac"]
        rec["kernel_sites"] = _kernel_table(sites, k_p)
    live = {"st": st, "hz": hz, "x": x, "gy": gy, "gen": gen, "act": act, "prog_on": prog_on, "prog_off": prog_off,
            "ms_on": ms_on, "ms_off": ms_off, "ms_c_on": ms_c_on, "us_per_tick": us_per_tick, "k_c": k_c, "cfg": cfg}
    rec["cpu_baseline"] = None
    return rec, live


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="bert_large_stage", help="the headline workload (value, ms_per_step)")
    ap.add_argument("--also", default="gpt2_1p5b_stage,large_layer_stage,tiny",
                    help="further workloads reported as sub-records under `workloads` (comma-separated, may be empty)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra-modes", action="store_true",
                    help="time modes A, B, C and the per-site pass of the headline workload only (profiler runs)")
    ap.add_argument("--profile-two-lanes", action="store_true",
                    help="run the per-site pass with FRC on (two lanes: a kernel's event time then "
                         "includes the time it shares the GPU with the other lane's kernels)")
    ap.add_argument("--roofline-only", action="store_true",
                    help="profiler aid: warm-up, then --steps iterations with an event pair around every launch, "
                         "nothing else; prints the roofline block and the per-site table of the workload")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one 256 MiB device copy (yardstick for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one stage on ONE GPU; --gpus %d is not supported (no collectives, no second "
              "GPU in this build)" % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_2204_12013_amd import binding as B, synth
    from paper_2204_12013_amd.harness import StageHarness
    if not torch.cuda.is_available():
        print("no GPU visible: the HIP path cannot run (there is no CPU fallback)", file=sys.stderr)
        return 3
    sc = synth.CONFIGS[args.workload]
    dev = torch.device("cuda:0")
    if args.roofline_only:
        rec, live = measure_core(B, synth, torch, sc, args.steps, args.warmup, args.profile_two_lanes, roofline_only=True)
        if args.calibration_copy:
            a = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
            b = torch.empty_like(a)
            a.fill_(1)
            torch.cuda.synchronize()
            B.bk_copy(a, b)
            torch.cuda.synchronize()
        live["st"].stage_destroy()
        print(json.dumps(rec))
        return 0
    rec, live = measure_core(B, synth, torch, sc, args.steps, args.warmup, args.profile_two_lanes)
    st, hz, x, gy, gen, act = (live[k] for k in ("st", "hz", "x", "gy", "gen", "act"))
    cfg, ms_on, ms_off, ms_c_on, us_per_tick, k_c = (live[k] for k in ("cfg", "ms_on", "ms_off", "ms_c_on", "us_per_tick", "k_c"))
    T, H, M = sc.tokens, sc.hidden, sc.M
    out = {"metric": "stage samples/s (FRC on/off), FRC overhead %, MFMA util vs bf16 peak",
           "value": rec["value"], "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": rec["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": rec["dtype"], "data": "synthetic"}
    out.update({k: v for k, v in rec.items() if k not in out})

    # The redundant-computation variants of the paper's microbenchmarks (Section 7.4, Table 4) on this
    # stage, in bubble mode: time of a failure-free iteration relative to running nothing redundant, and
    # the pause after a preemption (failover_merge until the lost state is rebuilt: BRC replay, plus,
    # with lazy FRC, the FRCs that were never run).
    if not args.no_extra_modes and sc.n_shadow > 0 and sc.stage_id < sc.P - 1:
        from paper_2204_12013_amd.harness import split_at_failure
        k_fail = min(5, M - 1)
        variants = {}
        for label, mode in (("LFLB", B.RC_LFLB), ("EFLB", B.RC_EFLB), ("EFEB", B.RC_EFEB)):
            sv = B.Stage(B.make_cfg(sc, rc_mode=mode), st.own_w, st.shadow_w)
            hv = StageHarness(sv, x, gz=gy, gy_table=gy)
            pv = sv.stage_schedule()

            def iters(n):
                hv.us_per_tick = us_per_tick
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(n):
                    hv.begin_iteration(zero_grads=True)
                    hv.run(pv)
                hv.sync()
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) * 1e3 / n
            iters(1)
            ms_v = iters(k_c)
            # preemption at micro-batch k_fail: time the part of the failover schedule that rebuilds lost state
            hv.us_per_tick = 0.0
            hv.begin_iteration(zero_grads=True)
            hv.run(split_at_failure(pv, k_fail))
            merged = sv.failover_merge(k_fail)
            first_group = _replay_end(B, merged)
            hv.sync()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            hv.run(merged[:first_group])
            hv.sync()
            torch.cuda.synchronize()
            pause = (time.perf_counter() - t0) * 1e3
            hv.run(merged[first_group:])
            hv.sync()
            variants[label] = {"ms_per_step": ms_v, "pause_ms": pause}
            sv.stage_destroy()
            del sv, hv
            torch.cuda.empty_cache()
        # How much of the eager FRC the bubbles hide depends on where the stage sits when the partition is
        # uneven (Section 5.2: later stages hold more layers and are slower, so early stages wait longer).
        # Same stage computation, timeline with the second half of the pipeline 25 % slower; one tick is
        # sized so that this stage's own forward + backward take their simulated number of ticks.
        by_stage = {}
        tfs = [4 if i < (sc.P + 1) // 2 else 5 for i in range(sc.P)]
        tbs = [2 * t for t in tfs]
        for sid in range(sc.P - 1):
            scs_ = sc.replace(stage_id=sid)
            sv = B.Stage(B.make_cfg(scs_), st.own_w, st.shadow_w)
            hv = StageHarness(sv, x, gz=gy, gy_table=gy)
            p_on = B.stage_program_uneven(sv.cfg, tfs, tbs)
            p_off = [i for i in p_on if i[0] != B.FRC]
            res = []
            for prog_ in (p_off, p_on):
                hv.us_per_tick = ms_off * 1e3 / (M * (tfs[sid] + tbs[sid]))
                for n_ in (1, 3):
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for _ in range(n_):
                        hv.begin_iteration(zero_grads=True)
                        hv.run(prog_)
                    hv.sync()
                    torch.cuda.synchronize()
                    t_ = (time.perf_counter() - t0) * 1e3 / n_
                res.append(t_)
            ticks = sum(i[3] for i in p_on if i[0] == B.BUBBLE)
            by_stage["stage_%d" % sid] = {"bubble_ticks": ticks, "ticks_per_fwd_bwd": tfs[sid] + tbs[sid],
                                          "ms_frc_off": res[0], "ms_frc_on": res[1],
                                          "frc_overhead_pct": 100.0 * (res[1] - res[0]) / res[0]}
            sv.stage_destroy()
            del sv, hv
            torch.cuda.empty_cache()
        out["frc_overhead_by_stage"] = {"timeline_ticks_fwd": tfs, "timeline_ticks_bwd": tbs, **by_stage}
        base = variants["LFLB"]["ms_per_step"]
        for v in variants.values():
            v["overhead_pct"] = 100.0 * (v["ms_per_step"] - base) / base
        out["rc_variants"] = {"mode": "simulated bubbles, %d iterations each, preemption at micro-batch %d" % (k_c, k_fail),
                              **variants}

    # Pure data parallelism (Section 5.2 "Support for Pure Data Parallelism", Section 7.6): the node holds the
    # whole model (here: the own layers) and the replica of a peer's model; there is no bubble, so eager FRC is
    # over-batching: the forward of the peer's minibatch beside the node's own.  The paper reports about 1.5x
    # the time for twice the batch on its GPUs.  Measured with the library's data-parallel mode: iteration
    # without redundancy, with eager FRC on the second lane, the merged node after the peer is lost (both
    # minibatches forward and backward), and the pause (BRC over the whole iteration's stash).
    if not args.no_extra_modes:
        from paper_2204_12013_amd.harness import split_at_failure
        scd = sc.replace(P=1, stage_id=0, n_shadow=sc.n_own)
        xn = [x[(k + 1) % M] for k in range(M)]
        dp = {}
        for label, mode in (("no_redundancy", B.RC_LFLB), ("eager_frc", B.RC_EFLB)):
            sd = B.Stage(B.make_cfg(scd, rc_mode=mode, data_parallel=1), st.own_w, st.own_w.clone())
            hd = StageHarness(sd, x, gz=gy, gy_table=gy, frc_in=xn)
            pd = sd.stage_schedule()
            _time_iters(torch, hd, pd, 1)
            dp[label] = _time_iters(torch, hd, pd, k_c)
            if mode == B.RC_EFLB:
                hd.begin_iteration(zero_grads=True)
                hd.run(split_at_failure(pd, M - 1))
                merged = sd.failover_merge(M - 1)
                first_group = _replay_end(B, merged)
                hd.sync()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                hd.run(merged[:first_group])
                hd.sync()
                torch.cuda.synchronize()
                dp["pause_ms"] = (time.perf_counter() - t0) * 1e3
                hd.run(merged[first_group:])
                hd.sync()
                hd.begin_iteration(zero_grads=True)      # the merged node's whole-iteration program is installed here
                pm = sd.stage_schedule()
                _time_iters(torch, hd, pm, 1)
                dp["merged_node"] = _time_iters(torch, hd, pm, k_c)
            sd.stage_destroy()
            del sd, hd
            torch.cuda.empty_cache()
        out["data_parallel"] = {"ms_per_step_no_redundancy": dp["no_redundancy"], "ms_per_step_eager_frc": dp["eager_frc"],
                                "eager_frc_time_ratio": dp["eager_frc"] / dp["no_redundancy"],
                                "ms_per_step_merged_node_two_minibatches": dp["merged_node"],
                                "merged_node_time_ratio": dp["merged_node"] / dp["no_redundancy"],
                                "pause_ms_peer_lost_at_end_of_iteration": dp["pause_ms"]}

    # Swap-out of the FRC results to host memory (Section 5.2; Section 7.4 puts the GPU-memory cost of eager
    # FRC at about 1.5x): the device keeps a ring of two shadow slots, every FRC's records go to pinned host
    # memory on a third stream and come back for BRC after a preemption.  Reported: iteration time with the
    # copies (no bubbles / simulated bubbles), the host-link rate they reach, the pause after a preemption,
    # and the device memory of the stage without redundancy, with the device-resident stash and with swap-out.
    if not args.no_extra_modes and sc.n_shadow > 0 and sc.stage_id < sc.P - 1:
        from paper_2204_12013_amd.harness import split_at_failure
        cfg_sw = B.make_cfg(sc, swap_slots=min(2, M))
        sz_sw = B.stage_query_sizes(cfg_sw)
        sz = st.sizes
        opt_own, opt_sh = int(sz.own_opt), int(sz.shadow_opt)
        mem_plain = int(sz.own_w + sz.own_g + sz.own_stash + sz.workspace) + opt_own
        mem_rc = mem_plain + int(sz.shadow_w + sz.shadow_g) + opt_sh
        mem = {"no_redundancy": mem_plain, "eager_frc_device_stash": mem_rc + int(sz.shadow_stash),
               "eager_frc_swap_out": mem_rc + int(sz_sw.shadow_stash), "host_pinned_swap_out": int(sz_sw.host_stash)}
        sw = {"device_bytes": mem,
              "device_memory_ratio": {"device_stash": mem["eager_frc_device_stash"] / mem_plain,
                                      "swap_out": mem["eager_frc_swap_out"] / mem_plain}}
        if int(sz_sw.host_stash) <= (8 << 30):      # timed only where the pinned buffer stays modest
            sv = B.Stage(cfg_sw, st.own_w, st.shadow_w)
            hv = StageHarness(sv, x, gz=gy, gy_table=gy)
            pv = sv.stage_schedule()

            def iters_sw(n, upt):
                hv.us_per_tick = upt
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(n):
                    hv.begin_iteration(zero_grads=True)
                    hv.run(pv)
                hv.sync()
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) * 1e3 / n
            iters_sw(1, 0.0)
            ms_sw = iters_sw(k_c, 0.0)
            ms_sw_c = iters_sw(k_c, us_per_tick)
            k_fail = min(5, M - 1)
            hv.us_per_tick = 0.0
            hv.begin_iteration(zero_grads=True)
            hv.run(split_at_failure(pv, k_fail))
            merged = sv.failover_merge(k_fail)
            first_group = _replay_end(B, merged)
            hv.sync()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            hv.run(merged[:first_group])
            hv.sync()
            torch.cuda.synchronize()
            pause = (time.perf_counter() - t0) * 1e3
            hv.run(merged[first_group:])
            hv.sync()
            sw.update({"ring_slots": int(cfg_sw.swap_slots), "ms_per_step_no_bubbles": ms_sw,
                       "ms_per_step_bubbles": ms_sw_c, "ms_per_step_device_stash_no_bubbles": ms_on,
                       "ms_per_step_device_stash_bubbles": ms_c_on,
                       "host_bytes_per_step": int(sz_sw.host_stash),
                       "device_to_host_GB/s_no_bubbles": int(sz_sw.host_stash) / (ms_sw * 1e-3) / 1e9,
                       "pause_ms_preemption_at_%d" % k_fail: pause})
            sv.stage_destroy()
            del sv, hv
            torch.cuda.empty_cache()
        out["swap_out"] = sw

    # The wrap-around stage (Section 5.1): the last stage with the LM head and the loss, holding the replica of
    # the first stage, whose FRC starts from token ids through the embedding.  Iteration time with and
    # without FRC, and the ends on their own (event pairs around each call): the head is three GEMMs of
    # 2 T H V flops (logits, weight gradient, input gradient) around the softmax cross-entropy, which reads
    # the logits once forward and rewrites them as their gradient backward.
    if not args.no_extra_modes and sc.n_shadow > 0 and sc.name in synth.VOCAB:
        import numpy as np
        from paper_2204_12013_amd.harness import WrapHarness
        V = synth.VOCAB[sc.name]
        scw = sc.replace(stage_id=sc.P - 1)
        cfg_w = B.make_cfg(scw, wrap=1)
        esz = B.ends_query_sizes(cfg_w, V)
        front_w = (torch.randn(int(esz.front_params), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(act)
        back_w = (torch.randn(int(esz.back_params), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(act)
        sw_ = B.Stage(cfg_w, st.own_w, st.shadow_w)
        en = B.Ends(cfg_w, V, front_w, back_w)
        rng = np.random.default_rng(sc.seed)
        ids = [torch.from_numpy(synth.zipf_ids(rng, V, T)).to(dev) for _ in range(M)]
        labels = [torch.from_numpy(synth.zipf_ids(rng, V, T)).to(dev) for _ in range(M)]
        torch.cuda.synchronize()
        hw = WrapHarness(sw_, en, x, ids, labels, gy)
        pw_on = sw_.stage_schedule()
        pw_off = [i for i in pw_on if i[0] != B.FRC]
        res = {}
        for label, prog_ in (("frc_on", pw_on), ("frc_off", pw_off)):
            for n_ in (1, k_c):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(n_):
                    hw.begin_iteration(zero_grads=True)
                    hw.run(prog_)
                hw.sync()
                torch.cuda.synchronize()
                res[label] = (time.perf_counter() - t0) * 1e3 / n_
        main = sw_.stream_main

        def timed(fn, reps=5):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            with torch.cuda.stream(main):
                e0.record()
                for _ in range(reps):
                    fn()
                e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        en.ends_begin_iteration()
        t_bf = timed(lambda: en.ends_back_fwd(hw.y[0], labels[0], hw.loss[0:1], main))
        t_bb = timed(lambda: (en.ends_back_fwd(hw.y[0], labels[0], hw.loss[0:1], main),
                              en.ends_back_bwd(hw.gy[0], main))) - t_bf
        t_ff = timed(lambda: en.ends_front_fwd(0, ids[0], hw.x0[0], main))
        t_fb = timed(lambda: (en.ends_front_fwd(0, ids[0], hw.x0[0], main),
                              en.ends_front_bwd(0, hw.dx0[0], main))) - t_ff
        head_flops = 2.0 * T * H * V
        out["wrap_around"] = {
            "vocab": V, "stage_id": sc.P - 1, "ms_per_step_frc_on": res["frc_on"], "ms_per_step_frc_off": res["frc_off"],
            "frc_overhead_pct_no_bubbles": 100.0 * (res["frc_on"] - res["frc_off"]) / res["frc_off"],
            "samples_per_s_frc_on": M * sc.micro_batch / (res["frc_on"] * 1e-3),
            "head_forward_ms": t_bf, "head_backward_ms": t_bb,
            "head_TFLOP/s": {"forward (1 GEMM + loss)": head_flops / (t_bf * 1e-3) / 1e12,
                             "backward (2 GEMMs + loss gradient)": 2 * head_flops / (t_bb * 1e-3) / 1e12},
            "embedding_forward_ms": t_ff, "embedding_backward_ms": t_fb}
        sw_.stage_destroy()
        en.ends_destroy()
        del sw_, en, hw, front_w, back_w
        torch.cuda.empty_cache()

    # Context for the roofline fraction: the stage's four forward GEMM shapes run stand-alone on operands
    # that are not cache-resident (a ring of buffer sets larger than the Infinity Cache, as inside an
    # iteration), this library's kernel beside the vendor GEMM that torch.matmul dispatches to.  The
    # vendor library is a yardstick for what the chip sustains at these sizes, nothing in the path uses it.
    if not args.no_extra_modes and sc.dtype == 1:
        ref = {}
        for name_, (N_, K_) in (("qkv", (3 * H, H)), ("attn_out", (H, H)), ("ffn1", (sc.ffn, H)), ("ffn2", (H, sc.ffn))):
            set_bytes = 2 * (T * K_ + K_ * N_ + T * N_)
            nb = max(2, min(64, int(1.2e9 // set_bytes)))
            Xs = [torch.randn(T, K_, device=dev, dtype=torch.float32).to(act) for _ in range(nb)]
            Ws = [(torch.randn(K_, N_, device=dev, dtype=torch.float32) * 0.02).to(act) for _ in range(nb)]
            Ys = [torch.empty(T, N_, device=dev, dtype=act) for _ in range(nb)]
            bias = torch.zeros(N_, device=dev, dtype=act)
            res = {}
            for who, fn in (("this_library", lambda i: B.bk_linear_fwd(Xs[i], Ws[i], bias, Ys[i], impl=2)),
                            ("vendor_via_torch", lambda i: torch.matmul(Xs[i], Ws[i], out=Ys[i]))):
                for i in range(nb):
                    fn(i)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                n_it = 3 * nb
                e0.record()
                for j in range(n_it):
                    fn(j % nb)
                e1.record()
                torch.cuda.synchronize()
                res[who] = 2.0 * T * N_ * K_ / (e0.elapsed_time(e1) * 1e-3 / n_it) / 1e12
            ref[name_] = {"M": T, "N": N_, "K": K_, "TFLOP/s": res}
            del Xs, Ws, Ys
        out["gemm_reference"] = ref
        torch.cuda.empty_cache()

    # the APPLY step (Adam over the own parameters) and the replica weight synchronisation, timed with
    # events on lane 0; algorithmic HBM bytes: 16 read + 14 written per parameter (fp32 gradient, master
    # weights and two moments in, the last three and the bf16 copy out); the synchronisation is a device
    # copy of the parameters and the optimizer state (2 + 12 bytes per parameter, read and written)
    st.stage_optimizer_init()
    n_own = int(st.sizes.layer_params) * sc.n_own
    n_sh = int(st.sizes.layer_params) * sc.n_shadow
    es = 2 if sc.dtype == 1 else 4
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    reps = 5
    st.stage_apply(1)
    st.stage_sync_replica(st.shadow_w, st.shadow_opt)          # self-copy: same traffic as from a neighbour's buffer
    st.stage_sync()
    with torch.cuda.stream(st.stream_main):
        ev[0].record()
        for i in range(reps):
            st.stage_apply(2 + i)
        ev[1].record()
        for i in range(reps):
            st.stage_sync_replica(st.shadow_w, st.shadow_opt)
        ev[2].record()
    st.stage_sync()
    t_adam = ev[0].elapsed_time(ev[1]) / reps
    t_sync = ev[1].elapsed_time(ev[2]) / reps
    out["apply_step"] = {"adam_ms": t_adam, "adam_GB/s": n_own * (28.0 + es) / (t_adam * 1e-3) / 1e9,
                         "adam_frac_of_hbm_peak": n_own * (28.0 + es) / (t_adam * 1e-3) / PEAK["hbm"],
                         "replica_sync_ms": t_sync,
                         "replica_sync_GB/s": 2.0 * n_sh * (12.0 + es) / (t_sync * 1e-3) / 1e9,
                         "parameters_own": n_own, "parameters_replica": n_sh}

    if args.calibration_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        a.fill_(1)
        torch.cuda.synchronize()
        B.bk_copy(a, b)
        torch.cuda.synchronize()
        del a, b
    st.stage_destroy()
    del st, hz, x, gy, live
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(sc)

    # The other workloads of the table, each with its own modes A / B / C, roofline and host baseline (fewer
    # steps where an iteration is long; the fp32 tiny workload is a correctness configuration: times only).
    others = {}
    for name in [n for n in args.also.split(",") if n and n != sc.name]:
        so = synth.CONFIGS[name]
        est_ms = ms_on * _iteration_flops(so, True) / _iteration_flops(sc, True)     # about 4 s of mode B each
        steps_o = max(3, min(args.steps, int(4000.0 / max(est_ms, 1e-3))))
        r, lv = measure_core(B, synth, torch, so, steps_o, max(1, min(args.warmup, 2)), args.profile_two_lanes)
        lv["st"].stage_destroy()
        del lv
        torch.cuda.empty_cache()
        if not args.no_cpu_baseline and so.dtype == 1:
            r["cpu_baseline"] = _cpu_baseline(so, seconds_budget=8.0)
        others[name] = r
    out["workloads"] = others
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
