"""Pins for oracle/schedule.py (integers only; no HIP path involved)."""
import itertools
import os

import pytest

from oracle import schedule as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_in_flight_counts_of_the_four_stage_example():
    """Section 5.2: in the 4-stage 1F1B figure the second stage holds 3 active
    micro-batches and the third holds 2."""
    assert S.own_slots(4, 1, 8) == 3 and S.own_slots(4, 2, 8) == 2
    # and the program really reaches, and never exceeds, that many
    for P, M in itertools.product(range(1, 6), range(1, 9)):
        for s in range(P):
            live = peak = 0
            for kind, _ in S.compute_order(P, s, M):
                live += 1 if kind == "F" else -1
                peak = max(peak, live)
                assert live >= 0
            assert live == 0 and peak == S.own_slots(P, s, M)


def test_every_microbatch_forward_then_backward_once():
    for P, M in itertools.product(range(1, 6), range(1, 9)):
        for s in range(P):
            seq = S.compute_order(P, s, M)
            assert sorted(seq) == sorted([("F", k) for k in range(M)] + [("B", k) for k in range(M)])
            for k in range(M):
                assert seq.index(("F", k)) < seq.index(("B", k))
            # one-forward-one-backward: after warm-up, kinds alternate
            w = S.warmup_depth(P, s, M)
            steady = seq[w:w + 2 * (M - w)]
            assert all(steady[i][0] == "FB"[i % 2] for i in range(len(steady)))


def test_uniform_pipeline_closed_form():
    """Equal stages: makespan (M+P-1)(tF+tB); each stage idles (P-1)(tF+tB),
    i.e. the textbook bubble fraction (P-1)/(M+P-1)."""
    for P, M, tf, tb in [(4, 8, 1, 2), (2, 3, 1, 1), (8, 16, 1, 2), (3, 3, 5, 7), (5, 2, 1, 2)]:
        start, end, makespan = S.timeline(P, M, tf, tb)
        assert makespan == (M + P - 1) * (tf + tb)
        for s in range(P):
            busy = sum(e - b for b, e in zip(start[s], end[s]))
            assert busy == M * (tf + tb)
            assert makespan - busy == (P - 1) * (tf + tb)


def test_bubble_of_the_unequal_pair_example():
    """Section 5.2 / Figure 9: a stage whose forward takes t next to a successor
    1.2x slower in both passes waits 0.6t at the barrier (t = 10 ticks, backward
    = 2 x forward)."""
    M = 6
    start, end, _ = S.timeline(2, M, [10, 12], [20, 24])
    seq = S.compute_order(2, 0, M)
    gaps = []
    for j in range(1, len(seq)):
        gaps.append((seq[j], start[0][j] - end[0][j - 1]))
    steady = [g for (kind, k), g in gaps if kind == "B" and 1 <= k <= M - 2]
    assert steady and all(g == 6 for g in steady), gaps


def test_hand_derived_timeline_of_the_bert_stage():
    rows = []
    makespan = None
    for line in open(os.path.join(GOLDEN, "cfg_bert_stage1_timeline.txt")):
        if line.startswith("# makespan"):
            makespan = int(line.split()[-1])
        if line.startswith("#") or not line.strip():
            continue
        kind, k, a, b = line.split()
        rows.append(((kind, int(k)), int(a), int(b)))
    start, end, mk = S.timeline(4, 8, 1, 2)
    seq = S.compute_order(4, 1, 8)
    assert mk == makespan == 33
    assert [(seq[j], start[1][j], end[1][j]) for j in range(len(seq))] == rows
    prog = S.stage_program(4, 1, 8, frc=True)
    bubbles = [a for op, _, _, a in prog if op == S.BUBBLE]
    assert bubbles == [1, 4, 1, 1, 2] and sum(bubbles) == 9
    # the bubbles after the first forward hold exactly the 8 ticks that 8 FRCs
    # of one tick each need
    assert sum(bubbles[1:]) == 8


def test_program_structure():
    for P, M in itertools.product(range(2, 6), range(1, 7)):
        for s in range(P):
            for frc in (False, True):
                prog = S.stage_program(P, s, M, frc=frc)
                ops = [i[0] for i in prog]
                assert ops[-3:] == [S.JOIN, S.ALLREDUCE, S.APPLY]
                C = S.own_slots(P, s, M)
                for j, (op, lane, k, arg) in enumerate(prog):
                    if op in (S.FWD, S.BWD):
                        assert lane == 0 and arg == k % C
                    if op == S.FRC:
                        assert lane == 1 and arg == k and prog[j - 1][:3] == (S.FWD, 0, k)
                    if op == S.SEND_ACT:
                        assert arg == s + 1 and s < P - 1
                    if op == S.RECV_ACT:
                        assert arg == s - 1 and s > 0
                assert ops.count(S.FRC) == (M if frc else 0)
                assert ops.count(S.FWD) == ops.count(S.BWD) == M
                assert ops.count(S.SEND_ACT) == ops.count(S.RECV_GRAD) == (M if s < P - 1 else 0)
                assert ops.count(S.RECV_ACT) == ops.count(S.SEND_GRAD) == (M if s > 0 else 0)
                # FRC(k) sits between FWD(k) and the send to the successor
                if frc and s < P - 1:
                    for k in range(M):
                        i_frc = prog.index((S.FRC, 1, k, k))
                        i_send = prog.index((S.SEND_ACT, 0, k, s + 1))
                        assert i_frc < i_send
                # total bubble time + busy time = makespan
                _, _, mk = S.timeline(P, M, 1, 2)
                assert sum(a for op, _, _, a in prog if op == S.BUBBLE) + 3 * M == mk


def _groups(prog):
    """Split at every comm->compute->comm change: a group = comm*, compute*."""
    comm = {S.RECV_ACT, S.SEND_ACT, S.RECV_GRAD, S.SEND_GRAD}
    comp = {S.FWD, S.BWD, S.FRC, S.BRC}
    groups, cur, seen_compute = [], [], False
    for ins in prog:
        if ins[0] in comm and seen_compute:
            groups.append(cur)
            cur, seen_compute = [], False
        if ins[0] in comp:
            seen_compute = True
        if ins[0] in comm or ins[0] in comp:
            cur.append(ins)
    if cur:
        groups.append(cur)
    return groups


def test_failover_merge_rules():
    """Section 5.2, rules (1)-(4) of the merged failover schedule."""
    comm = {S.RECV_ACT, S.SEND_ACT, S.RECV_GRAD, S.SEND_GRAD}
    for P, M in itertools.product(range(2, 6), range(1, 7)):
        for s in range(P - 1):
            for k_fail in range(M):
                b = S.lost_backwards(P, s, M, k_fail)
                w = S.warmup_depth(P, s, M)
                assert b == max(0, k_fail - w)
                pre = S.prefix_until_failure(P, s, M, k_fail)
                post = S.failover_program(P, s, M, k_fail)
                assert post[0] == (S.JOIN, 0, -1, k_fail)
                # rule 2: nothing is exchanged with the victim any more
                assert not [i for i in post if i[0] in comm and i[3] == s + 1]
                # after the failure everything runs on lane 0
                assert all(i[1] == 0 for i in post)
                # groups can only be told apart where every group has some communication left
                for g in (_groups(post) if (s > 0 and s + 2 < P) else []):
                    kinds = [i[0] in comm for i in g]
                    # rule 1: communication first
                    assert kinds == sorted(kinds, reverse=True)
                    # rule 3: the victim's external traffic (peer s+2) first
                    peers = [i[3] for i in g if i[0] in comm]
                    far = [p == s + 2 for p in peers]
                    assert far == sorted(far, reverse=True)
                    # rule 4: backward work before forward work
                    is_bwd = [i[0] in (S.BRC, S.BWD) for i in g if i[0] not in comm]
                    assert is_bwd == sorted(is_bwd, reverse=True)
                whole = pre + post
                for k in range(M):
                    assert sum(1 for i in whole if i[0] == S.FRC and i[2] == k) == 1
                    assert sum(1 for i in whole if i[0] == S.BRC and i[2] == k) == 1
                    assert sum(1 for i in whole if i[0] == S.FWD and i[2] == k) == 1
                    assert sum(1 for i in whole if i[0] == S.BWD and i[2] == k) == 1
                    i_brc = whole.index((S.BRC, 0, k, k))
                    i_bwd = [j for j, i in enumerate(whole) if i[0] == S.BWD and i[2] == k][0]
                    assert (i_brc < i_bwd) == (k >= b)      # replayed ones come after
                # shadow-gradient accumulation order is 0..M-1
                assert [i[2] for i in whole if i[0] == S.BRC] == list(range(M))
                if s + 2 < P:
                    sent = [i[2] for i in post if i[0] == S.SEND_ACT]
                    assert sent == list(range(k_fail, M))
                    assert [i[2] for i in post if i[0] == S.RECV_GRAD] == list(range(M))


def test_failover_example_of_the_bert_stage():
    post = S.failover_program(4, 1, 8, 5)
    text = S.fmt(post)
    assert text.startswith("JOIN RECV_GRAD(0) BRC(0) RECV_GRAD(1) BRC(1) RECV_GRAD(2) BRC(2) "
                           "SEND_ACT(5) RECV_GRAD(3) RECV_ACT(6) BRC(3) BWD(3) FWD(6) FRC(6) "
                           "SEND_ACT(6) RECV_GRAD(4) SEND_GRAD(3) RECV_ACT(7) BRC(4) BWD(4) FWD(7) FRC(7)")
    assert text.endswith("BRC(7) BWD(7) SEND_GRAD(7) JOIN ALLREDUCE APPLY")


def test_rc_variant_programs():
    """The three redundant-computation variants of Section 7.4 (Table 4) as instruction lists."""
    for P, M in itertools.product(range(2, 6), range(1, 6)):
        for s in range(P - 1):
            base = S.stage_program(P, s, M, rc=S.EFLB)
            assert base == S.stage_program(P, s, M, frc=True)
            lazy = S.stage_program(P, s, M, rc=S.LFLB)
            assert lazy == S.stage_program(P, s, M, frc=False) == [i for i in base if i[0] != S.FRC]
            eager = S.stage_program(P, s, M, rc=S.EFEB)
            # the eager-BRC program is the EFLB program plus, on lane 1, BRC(k) (and the receive of its
            # upstream gradient from the stage after the successor) ahead of the wait for BWD(k)
            assert [i for i in eager if i[1] == 0 or i[0] == S.FRC] == base
            extra = [i for i in eager if i[1] == 1 and i[0] != S.FRC]
            assert [i for i in extra if i[0] == S.BRC] == [(S.BRC, 1, k, k) for k in range(M)]
            assert len([i for i in extra if i[0] == S.RECV_GRAD]) == (M if s + 2 < P else 0)
            for k in range(M):
                i_brc = eager.index((S.BRC, 1, k, k))
                assert eager.index((S.FRC, 1, k, k)) < i_brc < eager.index((S.BWD, 0, k, k % S.own_slots(P, s, M)))
                nxt = [i for i in eager[i_brc + 1:] if i[0] != S.BUBBLE][0]
                assert nxt[0] in (S.SEND_ACT, S.SEND_GRAD, S.RECV_GRAD)     # issued before the stage waits
            for k_fail in range(M):
                b = S.lost_backwards(P, s, M, k_fail)
                f1 = S.failover_program(P, s, M, k_fail, rc=S.EFLB)
                f2 = S.failover_program(P, s, M, k_fail, rc=S.EFEB)
                f0 = S.failover_program(P, s, M, k_fail, rc=S.LFLB)
                n_replay = b * (2 if s + 2 < P else 1)
                assert f2 == f1[:1] + f1[1 + n_replay:]                     # no replay: BRC already ran
                # lazy FRC: every FRC of the iteration happens after the failure, each before its BRC
                whole = S.prefix_until_failure(P, s, M, k_fail, rc=S.LFLB) + f0
                for k in range(M):
                    assert sum(1 for i in whole if i[0] == S.FRC and i[2] == k) == 1
                    assert sum(1 for i in whole if i[0] == S.BRC and i[2] == k) == 1
                    assert whole.index((S.FRC, 0, k, k)) < whole.index((S.BRC, 0, k, k))
                assert [i[2] for i in whole if i[0] == S.BRC] == list(range(M))
                rest = lambda f: [i for i in f if i[0] != S.FRC or i[2] > k_fail]
                assert rest(f0) == rest(f1)
                whole2 = S.prefix_until_failure(P, s, M, k_fail, rc=S.EFEB) + f2
                assert [i[2] for i in whole2 if i[0] == S.BRC] == list(range(M))


def test_wrap_around_victim_progress_hand_derived():
    """The last stage shadows the first (Section 5.1).  Where the first stage stands when the last one
    has finished FWD(k_fail), worked out by hand on the zero-latency timeline with forward 1 / backward 2
    ticks: P=4: the last stage runs F(k) at 3+3k, so F(2) ends at 10; the first stage ran F0..F2 at 0,1,2,
    F3 at 3 and waits for its first backward until 10.  P=2, k_fail=1: F1 of stage 1 ends at 5, stage 0
    did F0, F1 and is inside B0 (4..6).  P=2, k_fail=3: F3 of stage 1 ends at 11; stage 0 finished B0 (6)
    and B1 (9), B2 runs 10..12."""
    assert S.wrap_victim_progress(4, 8, 2) == (4, 0)
    assert S.wrap_victim_progress(2, 4, 1) == (2, 0)
    assert S.wrap_victim_progress(2, 4, 3) == (4, 2)


def test_wrap_around_failover_program_invariants():
    for P, M in itertools.product(range(2, 7), [1, 2, 3, 5, 8]):
        for k_fail in range(M):
            for tf, tb in ((1, 2), (2, 3)):
                prog = S.wrap_failover_program(P, M, k_fail, tf, tb)
                nf, nb = S.wrap_victim_progress(P, M, k_fail, tf, tb)
                assert nf > k_fail and nb <= k_fail           # the victim is ahead forwards, behind backwards
                pos = {}
                for i, (op, lane, k, arg) in enumerate(prog):
                    assert lane == 0
                    if op in (S.FWD, S.BWD, S.FRC, S.BRC):
                        assert (op, k) not in pos
                        pos[(op, k)] = i
                assert prog[0] == (S.JOIN, 0, -1, k_fail) and prog[-3:] == [(S.JOIN, 0, -1, -1), (S.ALLREDUCE, 0, -1, 0), (S.APPLY, 0, -1, 0)]
                # the shadow's own remaining work, the victim's forwards beyond k_fail, every victim backward
                assert sorted(k for (op, k) in pos if op == S.FWD) == list(range(k_fail + 1, M))
                assert sorted(k for (op, k) in pos if op == S.BWD) == list(range(k_fail, M))
                assert sorted(k for (op, k) in pos if op == S.FRC) == list(range(k_fail + 1, M))
                assert sorted(k for (op, k) in pos if op == S.BRC) == list(range(M))
                # replayed backwards come first, in order
                assert [ins[2] for ins in prog if ins[0] == S.BRC][:nb] == list(range(nb))
                for k in range(M):
                    if k > k_fail:
                        assert pos[(S.FRC, k)] < pos[(S.BRC, k)] and pos[(S.FWD, k)] < pos[(S.BWD, k)]
                        assert pos[(S.FRC, k)] < pos[(S.FWD, k)]      # the front of the pipeline runs first
                    if k >= k_fail:
                        assert pos[(S.BWD, k)] < pos[(S.BRC, k)]      # the gradient travels back to the front
                # outputs of the victim's forwards go to the second stage only if it never got them
                sends = sorted(ins[2] for ins in prog if ins[0] == S.SEND_ACT)
                assert sends == ([k for k in range(k_fail + 1, M) if k >= nf] if P > 2 else [])
                recv_g = sorted(ins[2] for ins in prog if ins[0] == S.RECV_GRAD)
                assert recv_g == (list(range(M)) if P > 2 else [])
                for ins in prog:
                    if ins[0] in (S.SEND_ACT, S.RECV_GRAD):
                        assert ins[3] == 1
                    if ins[0] in (S.RECV_ACT, S.SEND_GRAD):
                        assert ins[3] == P - 2 and P > 2
                    if ins[0] in (S.FWD, S.BWD):
                        assert ins[3] == ins[2] % S.own_slots(P, P - 1, M)
                # own slot discipline: at most one forward in flight on the last stage
                live = {k_fail}
                for op, _, k, _ in prog:
                    if op == S.FWD:
                        assert not live
                        live.add(k)
                    elif op == S.BWD:
                        live.remove(k)


def test_merged_program_structure():
    """Rules 1-4 of Section 5.2 on the merged stage's whole iteration: no traffic between victim and
    shadow is left, every group leads with its communication (the victim's external traffic before the
    shadow's own), backward work precedes forward work, every micro-batch has exactly one FWD, FRC,
    BRC and BWD, and the order of the own computations is the stage's 1F1B order."""
    for P in range(2, 7):
        for s in range(P - 1):
            for M in (1, 2, 3, 5, 8):
                prog = S.merged_program(P, s, M)
                assert prog[-3:] == [(S.JOIN, 0, -1, -1), (S.ALLREDUCE, 0, -1, 0), (S.APPLY, 0, -1, 0)]
                assert all(lane == 0 for _, lane, _, _ in prog)
                assert not any(op in (S.SEND_ACT, S.RECV_GRAD) and arg == s + 1 for op, _, _, arg in prog)
                for op in (S.FWD, S.FRC, S.BRC, S.BWD):
                    assert sorted(k for o, _, k, _ in prog if o == op) == list(range(M))
                own = [("F" if op == S.FWD else "B", k) for op, _, k, _ in prog if op in (S.FWD, S.BWD)]
                assert own == S.compute_order(P, s, M)
                pos = {(op, k): i for i, (op, _, k, _) in enumerate(prog)}
                for k in range(M):
                    assert pos[(S.FWD, k)] < pos[(S.FRC, k)] < pos[(S.BRC, k)] < pos[(S.BWD, k)]
                    if s + 2 < P:      # the victim's external traffic exists and brackets its work
                        assert pos[(S.FRC, k)] < pos[(S.SEND_ACT, k)] < pos[(S.RECV_GRAD, k)] < pos[(S.BRC, k)]
                    else:
                        assert (S.SEND_ACT, k) not in pos and (S.RECV_GRAD, k) not in pos
                    if s > 0:
                        assert pos[(S.RECV_ACT, k)] < pos[(S.FWD, k)] and pos[(S.BWD, k)] < pos[(S.SEND_GRAD, k)]
                # inside a run of instructions between computations, communication never follows computation
                comm = (S.SEND_ACT, S.RECV_ACT, S.SEND_GRAD, S.RECV_GRAD)
                groups, cur = [], []
                for ins in prog[:-3]:
                    if ins[0] in comm and cur and cur[-1][0] not in comm:
                        groups.append(cur)
                        cur = []
                    cur.append(ins)
                groups.append(cur)
                for grp in groups if s + 2 < P else []:     # (groups show only where every one of them has traffic)
                    ops = [i[0] for i in grp if i[0] not in comm]
                    if S.BWD in ops and S.FWD in ops:
                        assert ops.index(S.BWD) < ops.index(S.FWD)          # rule 4
                    far = [i for i, ins in enumerate(grp) if ins[0] in comm and ins[3] == s + 2]
                    near = [i for i, ins in enumerate(grp) if ins[0] in comm and ins[3] == s - 1]
                    if far and near:
                        assert max(far) < min(near)                            # rule 3
    # the failover schedule's last part, started at the first computation, is the same list
    full = S.merged_program(4, 1, 8)
    tail = S.failover_program(4, 1, 8, 0)
    i = next(i for i, ins in enumerate(tail) if ins[0] == S.BRC and ins[2] == 0)
    j = next(i for i, ins in enumerate(full) if ins[0] == S.BRC and ins[2] == 0)
    assert [ins for ins in tail[i:] if ins[0] not in (S.SEND_ACT,)] == [ins for ins in full[j:] if ins[0] not in (S.SEND_ACT,)]


def test_data_parallel_programs():
    """Pure data parallelism (Section 5.2): one node, no bubbles, no communication before the
    all-reduce; eager FRC sits beside every forward."""
    M = 5
    prog = S.stage_program(1, 0, M)
    assert [(op, lane, k) for op, lane, k, _ in prog[:-3]] == [
        t for k in range(M) for t in ((S.FWD, 0, k), (S.FRC, 1, k), (S.BWD, 0, k))]
    assert not any(op == S.BUBBLE for op, _, _, _ in prog)
    assert S.own_slots(1, 0, M) == 1
    merged = S.merged_program(1, 0, M)
    assert [(op, k) for op, _, k, _ in merged[:-3]] == [
        (S.FWD, 0), (S.FRC, 0)] + [t for k in range(M - 1) for t in ((S.BRC, k), (S.BWD, k), (S.FWD, k + 1), (S.FRC, k + 1))
                                   ] + [(S.BRC, M - 1), (S.BWD, M - 1)]
    for k_fail in range(M):
        f = S.failover_program(1, 0, M, k_fail, data_parallel=True)
        assert f[0] == (S.JOIN, 0, -1, k_fail)
        assert [k for op, _, k, _ in f if op == S.BRC] == list(range(M))
        assert [k for op, _, k, _ in f if op == S.FRC] == list(range(k_fail + 1, M))


def test_wrap_merged_program_structure():
    for P in (2, 3, 4, 6):
        for M in (1, 3, 4, 8):
            prog = S.wrap_merged_program(P, M)
            for op in (S.FWD, S.FRC, S.BRC, S.BWD):
                assert sorted(k for o, _, k, _ in prog if o == op) == list(range(M))
            pos = {(op, k): i for i, (op, _, k, _) in enumerate(prog)}
            for k in range(M):
                # the first stage's forward of a micro-batch precedes the last stage's, its backward follows it
                assert pos[(S.FRC, k)] < pos[(S.FWD, k)] < pos[(S.BWD, k)] < pos[(S.BRC, k)]
            own = [("F" if op == S.FWD else "B", k) for op, _, k, _ in prog if op in (S.FWD, S.BWD)]
            vic = [("F" if op == S.FRC else "B", k) for op, _, k, _ in prog if op in (S.FRC, S.BRC)]
            assert own == S.compute_order(P, P - 1, M) and vic == S.compute_order(P, 0, M)
            # the failover schedule for a loss at the very first micro-batch ends the same way
            f = S.wrap_failover_program(P, M, 0)
            last = lambda p: [i for i in p if i[0] in (S.FWD, S.BWD, S.FRC, S.BRC)][-2 * M:]
            assert last(f) == last(prog)
