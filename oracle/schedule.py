"""Reference slot schedule of one Bamboo stage (oracle; test infrastructure).

Integers only.  Follows the paper's description in prose (its figures are not
available): the 1F1B schedule of Section 2, instruction groups and the static
per-stage schedule of Sections 4 and 5.2, eager FRC placed before the stage
talks to its successor (Section 5.2 "Scheduling"), and the four merge rules of
the failover schedule (Section 5.2 "Lazy BRC and Recovery").

An instruction is a tuple (op, lane, mb, arg):
  op    one of the codes below
  lane  0 = main stream, 1 = FRC stream
  mb    micro-batch id, -1 when the instruction has none
  arg   FWD/BWD: own stash slot (mb mod C_own); FRC/BRC: shadow stash slot (mb);
        comm ops: id of the peer stage; BUBBLE: ticks; JOIN: last FRC waited for
        (-1: all); otherwise 0
"""

RECV_ACT, SEND_ACT, RECV_GRAD, SEND_GRAD, FWD, BWD, FRC, BRC, BUBBLE, JOIN, ALLREDUCE, APPLY = range(12)

# Redundant-computation variants compared in the paper's microbenchmarks (Section 7.4, Table 4):
# lazy FRC + lazy BRC, eager FRC + lazy BRC (Bamboo's choice), eager FRC + eager BRC.
LFLB, EFLB, EFEB = 0, 1, 2
OP_NAMES = ("RECV_ACT", "SEND_ACT", "RECV_GRAD", "SEND_GRAD", "FWD", "BWD",
            "FRC", "BRC", "BUBBLE", "JOIN", "ALLREDUCE", "APPLY")


def warmup_depth(P, s, M):
    """Forwards a 1F1B stage runs before its first backward, minus one."""
    return min(P - 1 - s, M)


def own_slots(P, s, M):
    """Peak number of in-flight micro-batches of stage s (Section 5.2: with four
    stages, the second stage holds 3 and the third holds 2)."""
    return min(P - s, M)


def compute_order(P, s, M):
    """1F1B compute sequence of stage s as a list of ('F'|'B', k)."""
    w = warmup_depth(P, s, M)
    seq = [("F", k) for k in range(w)]
    for i in range(M - w):
        seq.append(("F", w + i))
        seq.append(("B", i))
    seq += [("B", k) for k in range(M - w, M)]
    return seq


def timeline(P, M, tick_F, tick_B):
    """Simulate all P stages with zero communication latency.

    tick_F / tick_B: int or per-stage sequences.  Returns (start, end, makespan)
    where start[s][j], end[s][j] are the times of the j-th compute instruction of
    stage s.  A forward waits for the same micro-batch's forward on the previous
    stage; a backward waits for its backward on the next stage; instructions of a
    stage run in program order.
    """
    tf = [tick_F] * P if isinstance(tick_F, int) else list(tick_F)
    tb = [tick_B] * P if isinstance(tick_B, int) else list(tick_B)
    seqs = [compute_order(P, s, M) for s in range(P)]
    start = [[None] * len(q) for q in seqs]
    end = [[None] * len(q) for q in seqs]
    done = {}                      # (kind, stage, k) -> end time
    pos = [0] * P
    clock = [0] * P
    progressed = True
    while progressed:
        progressed = False
        for s in range(P):
            while pos[s] < len(seqs[s]):
                kind, k = seqs[s][pos[s]]
                if kind == "F":
                    dep = done.get(("F", s - 1, k)) if s > 0 else 0
                    dur = tf[s]
                else:
                    dep = done.get(("B", s + 1, k)) if s < P - 1 else 0
                    dur = tb[s]
                if dep is None:
                    break
                t0 = max(clock[s], dep)
                start[s][pos[s]] = t0
                end[s][pos[s]] = t0 + dur
                clock[s] = t0 + dur
                done[(kind, s, k)] = t0 + dur
                pos[s] += 1
                progressed = True
    assert all(pos[s] == len(seqs[s]) for s in range(P)), "1F1B deadlock"
    return start, end, max(clock)


def _head_comm(prev, cur, P, s):
    """Communication instructions at the head of cur's group: first the send of
    what the previous compute produced, then the receive cur needs."""
    out = []
    if prev is not None:
        kind, k = prev
        if kind == "F" and s < P - 1:
            out.append((SEND_ACT, 0, k, s + 1))
        if kind == "B" and s > 0:
            out.append((SEND_GRAD, 0, k, s - 1))
    if cur is not None:
        kind, k = cur
        if kind == "F" and s > 0:
            out.append((RECV_ACT, 0, k, s - 1))
        if kind == "B" and s < P - 1:
            out.append((RECV_GRAD, 0, k, s + 1))
    return out


def stage_program(P, s, M, frc=True, tick_F=1, tick_B=2, bubbles=True, rc=None):
    """Instruction list of stage s for one iteration (no failure).

    rc (overrides frc): LFLB emits no redundant computation at all; EFLB emits FRC(k) on lane 1
    right after FWD(k); EFEB additionally emits BRC(k) on lane 1 as soon as the upstream gradient
    of the successor's layers exists, i.e. where the stage starts to wait for the successor's
    backward of micro-batch k (the receive from the stage after the successor comes with it).
    """
    if rc is None:
        rc = EFLB if frc else LFLB
    frc = rc != LFLB
    seq = compute_order(P, s, M)
    C = own_slots(P, s, M)
    start, end, makespan = timeline(P, M, tick_F, tick_B)
    prog, prev, clock = [], None, 0
    for j, cur in enumerate(seq):
        gap = start[s][j] - clock
        kind, k = cur
        if rc == EFEB and kind == "B" and s < P - 1:
            if s + 2 < P:
                prog.append((RECV_GRAD, 1, k, s + 2))
            prog.append((BRC, 1, k, k))
        if bubbles and gap > 0:
            prog.append((BUBBLE, 0, -1, gap))
        prog += _head_comm(prev, cur, P, s)
        if kind == "F":
            prog.append((FWD, 0, k, k % C))
            if frc:
                prog.append((FRC, 1, k, k))
        else:
            prog.append((BWD, 0, k, k % C))
        clock = end[s][j]
        prev = cur
    tail = makespan - clock
    prog += _head_comm(prev, None, P, s)
    if bubbles and tail > 0:
        prog.append((BUBBLE, 0, -1, tail))
    prog += [(JOIN, 0, -1, -1), (ALLREDUCE, 0, -1, 0), (APPLY, 0, -1, 0)]
    return prog


def lost_backwards(P, s, M, k_fail):
    """Backwards stage s (and hence its successor) had completed when the send
    of micro-batch k_fail's activation to the successor fails."""
    seq = compute_order(P, s, M)
    j = seq.index(("F", k_fail))
    return sum(1 for kind, _ in seq[:j] if kind == "B")


def prefix_until_failure(P, s, M, k_fail, frc=True, tick_F=1, tick_B=2, bubbles=True, rc=None):
    """The part of the normal program that ran before the failure was detected:
    everything up to and including FWD(k_fail) and its FRC."""
    prog = stage_program(P, s, M, frc, tick_F, tick_B, bubbles, rc)
    last = max(i for i, ins in enumerate(prog)
               if ins[2] == k_fail and ins[0] in (FWD, FRC))
    return prog[:last + 1]


def _merge_groups(rest, C, s, has_far, unsent_act):
    """Rules (1)-(4) of Section 5.2 over the 1F1B computations in `rest`: the instruction list of the
    shadow stage doing its own work and the victim's, up to (not including) the closing
    JOIN / ALLREDUCE / APPLY.  A backward opens a group and the forward that follows it in 1F1B order
    joins that group; inside a group communication comes first -- the victim's external traffic (with
    the stage after it, if has_far) before the shadow's own (with stage s-1, if s > 0), traffic between
    victim and shadow is gone --, then backward work (victim's BRC, own BWD), then forward work (own
    FWD, victim's FRC, now on lane 0).  unsent_act: FRC outputs the stage after the victim still has
    to be sent when the list starts."""
    prog = []
    groups = []
    for item in rest:
        if item[0] == "B" or not groups or groups[-1][-1][0] == "F":
            groups.append([item])
        else:
            groups[-1].append(item)
    unsent_act = list(unsent_act)           # FRC outputs the far stage has not got
    unsent_grad = []                        # own input-gradients not yet sent back
    for grp in groups + [[]]:
        # victim's external communication first
        if has_far:
            prog += [(SEND_ACT, 0, k, s + 2) for k in unsent_act]
        unsent_act = []
        for kind, k in grp:
            if kind == "B" and has_far:
                prog.append((RECV_GRAD, 0, k, s + 2))
        # then the shadow's own
        if s > 0:
            prog += [(SEND_GRAD, 0, k, s - 1) for k in unsent_grad]
        unsent_grad = []
        for kind, k in grp:
            if kind == "F" and s > 0:
                prog.append((RECV_ACT, 0, k, s - 1))
        # compute: backward (victim's then own), then forward (own then victim's)
        for kind, k in grp:
            if kind == "B":
                prog.append((BRC, 0, k, k))
                prog.append((BWD, 0, k, k % C))
                unsent_grad.append(k)
        for kind, k in grp:
            if kind == "F":
                prog.append((FWD, 0, k, k % C))
                prog.append((FRC, 0, k, k))
                unsent_act.append(k)
    return prog


def failover_program(P, s, M, k_fail, rc=EFLB, data_parallel=False):
    """Failover schedule of shadow stage s after its successor s+1 is lost while
    stage s tries to send it the activation of micro-batch k_fail.

    rc = EFLB is the paper's design and the description below.  With EFEB step (ii) is empty
    (BRC of those micro-batches already ran, eagerly).  With LFLB nothing redundant has been
    computed yet: step (ii) runs FRC before each BRC, and the FRC of the micro-batches the
    victim had forwarded but not yet back-propagated follows before step (iii) -- this is the
    longer pause that eager FRC avoids (Section 7.4).

    (i)   wait for the FRC stream up to FRC(k_fail);
    (ii)  replay: BRC over the micro-batches whose successor-side backward had
          already run (their weight-gradient contributions died with the victim);
    (iii) the rest of stage s's 1F1B program with the victim's groups merged in:
          communication first, victim<->shadow traffic removed, the victim's
          external traffic before the shadow's, backward work before forward work.

    data_parallel (Section 5.2, "Support for Pure Data Parallelism"): the node holds the whole model
    (P = 1) and the victim is the node whose replica it keeps, working through the same schedule on
    its own minibatch; the loss is noticed after FWD(k_fail) and its FRC as above.  Nothing is
    exchanged between the two before the all-reduce, so the schedule has no communication at all.
    """
    if data_parallel:
        assert P == 1 and s == 0 and 0 <= k_fail < M and rc != EFEB
    else:
        assert 0 <= s < P - 1 and 0 <= k_fail < M
    seq = compute_order(P, s, M)
    C = own_slots(P, s, M)
    has_far = s + 2 < P                     # the victim had a successor of its own
    b = lost_backwards(P, s, M, k_fail)
    prog = [(JOIN, 0, -1, k_fail)]
    if rc != EFEB:
        for k in range(b):
            if has_far:
                prog.append((RECV_GRAD, 0, k, s + 2))
            if rc == LFLB:
                prog.append((FRC, 0, k, k))
            prog.append((BRC, 0, k, k))
    if rc == LFLB:
        prog += [(FRC, 0, k, k) for k in range(b, k_fail + 1)]
    rest = seq[seq.index(("F", k_fail)) + 1:]
    prog += _merge_groups(rest, C, s, has_far, [k_fail])
    prog += [(JOIN, 0, -1, -1), (ALLREDUCE, 0, -1, 0), (APPLY, 0, -1, 0)]
    return prog


def merged_program(P, s, M):
    """A whole iteration of the stage once it has taken over its successor's layers (Section 5.2:
    until the pipeline is reconfigured the shadow node executes all of the victim's instructions):
    the stage's own 1F1B order, every computation merged with the victim's of the same micro-batch
    under the same four rules as the failover schedule -- which is that schedule's part (iii) started
    at the first computation, with nothing to join and nothing to replay.  No bubbles are simulated.
    With P = 1 this is the merged node of pure data parallelism (both minibatches, no communication)."""
    assert (0 <= s < P - 1 or (P == 1 and s == 0)) and M >= 1
    prog = _merge_groups(compute_order(P, s, M), own_slots(P, s, M), s, s + 2 < P, [])
    return prog + [(JOIN, 0, -1, -1), (ALLREDUCE, 0, -1, 0), (APPLY, 0, -1, 0)]


def fmt(prog):
    return " ".join(
        OP_NAMES[op] + ("" if mb < 0 else "(%d)" % mb) +
        ("[%d]" % arg if op in (BUBBLE,) else "") + ("@1" if lane else "")
        for op, lane, mb, arg in prog)


# ---- wrap-around: the last stage shadows the first (Section 5.1) ------------------

def wrap_victim_progress(P, M, k_fail, tick_F=1, tick_B=2):
    """State of the first stage when the last stage finishes FWD(k_fail) in the failure-free
    timeline: (number of forwards, number of backwards) the first stage has completed by then.
    Both run in micro-batch order, so the counts say which ones."""
    start, end, _ = timeline(P, M, tick_F, tick_B)
    last = compute_order(P, P - 1, M)
    t_star = end[P - 1][last.index(("F", k_fail))]
    first = compute_order(P, 0, M)
    nf = sum(1 for j, (kind, _) in enumerate(first) if kind == "F" and end[0][j] <= t_star)
    nb = sum(1 for j, (kind, _) in enumerate(first) if kind == "B" and end[0][j] <= t_star)
    return nf, nb


def wrap_failover_program(P, M, k_fail, tick_F=1, tick_B=2, rc=EFLB):
    """Failover schedule of the last stage (s = P-1) after the first stage, whose replica it holds,
    is lost.  The last stage notices right after FWD(k_fail) and its FRC, as a middle stage does.

    The two merged stages are the two ends of the pipeline, so unlike the adjacent case no
    traffic between them becomes internal (unless P = 2, where each is the other's only
    neighbour and all of it does).  The schedule:
      (i)   wait for the FRC stream up to FRC(k_fail);
      (ii)  replay BRC over the micro-batches whose first-stage backward had run (their gradient
            contributions died with the victim); the second stage sends their gradients again;
      (iii) everything else either stage still has to do, ordered by its start time in the
            failure-free timeline (a valid order: whatever a computation depends on started
            earlier there), ties broken as in the adjacent case -- backward work before forward
            work, the victim's before the shadow's own.  The victim's forwards are FRCs on the
            samples the last node fetches itself; they are all still to do beyond k_fail, and
            their outputs go to the second stage unless the victim had delivered them already.
    Communication is emitted as in the normal program: the send of what the previous computation
    of a stage produced, then the receive the next one needs, right before it.

    rc = LFLB (Section 7.4's lazy variant on this stage): nothing redundant has run, so step (ii)
    runs FRC before every BRC, and the forwards the victim had done but not yet back-propagated
    (all delivered to the second stage already: the last stage cannot be at micro-batch k_fail
    before the first has forwarded it) are run again right after, for their intermediates.
    """
    assert P >= 2 and 0 <= k_fail < M and rc in (LFLB, EFLB)
    s = P - 1
    C = own_slots(P, s, M)
    start, end, _ = timeline(P, M, tick_F, tick_B)
    nf, nb = wrap_victim_progress(P, M, k_fail, tick_F, tick_B)
    far = P > 2                               # the victim's neighbour is not the shadow itself
    prog = [(JOIN, 0, -1, k_fail)]
    for k in range(nb):
        if far:
            prog.append((RECV_GRAD, 0, k, 1))
        if rc == LFLB:
            prog.append((FRC, 0, k, k))
        prog.append((BRC, 0, k, k))
    if rc == LFLB:
        prog += [(FRC, 0, k, k) for k in range(nb, k_fail + 1)]
    own = compute_order(P, s, M)
    j0 = own.index(("F", k_fail)) + 1
    items = []                                # (start time, 0 backward / 1 forward, 0 victim / 1 own, kind, k)
    for j in range(j0, len(own)):
        kind, k = own[j]
        items.append((start[s][j], 0 if kind == "B" else 1, 1, kind, k))
    for j, (kind, k) in enumerate(compute_order(P, 0, M)):
        if (kind == "F" and k > k_fail) or (kind == "B" and k >= nb):
            items.append((start[0][j], 0 if kind == "B" else 1, 0, kind, k))
    items.sort()
    pending = []                              # sends owed for computations already emitted
    for _, _, is_own, kind, k in items:
        prog += pending
        pending = []
        if is_own:
            if kind == "F":
                if far:
                    prog.append((RECV_ACT, 0, k, s - 1))
                prog.append((FWD, 0, k, k % C))
            else:
                prog.append((BWD, 0, k, k % C))
                if far:
                    pending.append((SEND_GRAD, 0, k, s - 1))
        else:
            if kind == "F":
                prog.append((FRC, 0, k, k))
                if far and k >= nf:
                    pending.append((SEND_ACT, 0, k, 1))
            else:
                if far:
                    prog.append((RECV_GRAD, 0, k, 1))
                prog.append((BRC, 0, k, k))
    prog += pending
    prog += [(JOIN, 0, -1, -1), (ALLREDUCE, 0, -1, 0), (APPLY, 0, -1, 0)]
    return prog


def wrap_merged_program(P, M, tick_F=1, tick_B=2):
    """A whole iteration of the last stage once it has taken over the first stage's layers: every
    computation of both stages, ordered as in part (iii) of wrap_failover_program (start time on the
    failure-free timeline; backward before forward, the victim's before the shadow's own), with the
    same placement of the communication.  Nothing to join, nothing to replay."""
    assert P >= 2 and M >= 1
    s = P - 1
    C = own_slots(P, s, M)
    start, end, _ = timeline(P, M, tick_F, tick_B)
    far = P > 2
    items = []
    for j, (kind, k) in enumerate(compute_order(P, s, M)):
        items.append((start[s][j], 0 if kind == "B" else 1, 1, kind, k))
    for j, (kind, k) in enumerate(compute_order(P, 0, M)):
        items.append((start[0][j], 0 if kind == "B" else 1, 0, kind, k))
    items.sort()
    prog, pending = [], []
    for _, _, is_own, kind, k in items:
        prog += pending
        pending = []
        if is_own:
            if kind == "F":
                if far:
                    prog.append((RECV_ACT, 0, k, s - 1))
                prog.append((FWD, 0, k, k % C))
            else:
                prog.append((BWD, 0, k, k % C))
                if far:
                    pending.append((SEND_GRAD, 0, k, s - 1))
        else:
            if kind == "F":
                prog.append((FRC, 0, k, k))
                if far:
                    pending.append((SEND_ACT, 0, k, 1))
            else:
                if far:
                    prog.append((RECV_GRAD, 0, k, 1))
                prog.append((BRC, 0, k, k))
    prog += pending
    prog += [(JOIN, 0, -1, -1), (ALLREDUCE, 0, -1, 0), (APPLY, 0, -1, 0)]
    return prog
