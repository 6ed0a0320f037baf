"""The neighbours of one Stage: buffer tables and the communication hook for the library's
instruction-list interpreter (stage_run).

The stage before (s-1) is a table of inputs x_k, the stage after the successor
(s+2) a table of upstream gradients g_z_k, both pre-staged in device memory
(they replace RECV_ACT / RECV_GRAD).  The successor (s+1) is either absent
(benchmark: g_y_k comes from a table) or simulated by a second Stage object
running the replica's parameter values as its own layers, with its own stash
and gradient buffer, until it is "preempted".  No arithmetic happens here and no
instruction is interpreted here: the list goes to stage_run, which issues every
computation; this side answers the communication instructions.
"""
from . import binding as B


class StageHarness:
    def __init__(self, stage, x, gz, successor=None, gy_table=None, us_per_tick=0.0, adam=None, frc_in=None):
        self.st = stage
        self.x, self.gz = x, gz
        self.frc_in = frc_in      # inputs of FRC where they are not the stage's own outputs (data-parallel peer)
        self.succ = successor
        self.gy_table = gy_table
        self.us_per_tick = us_per_tick
        self.adam = adam          # dict of Adam hyper-parameters: APPLY then runs the optimizer step
        self.step = 0
        M = stage.cfg.M
        self.y = [stage.new_act() for _ in range(M)]
        self.gx = [stage.new_act() for _ in range(M)]
        self.z_frc = [stage.new_act() for _ in range(M)] if stage.cfg.n_shadow > 0 else None
        self.gy = list(gy_table) if gy_table is not None else [stage.new_act() for _ in range(M)]
        self.gy_replay = {}
        self.bwd_done = set()
        if successor is not None:
            self.z_succ = [stage.new_act() for _ in range(M)]
            self.succ_fwd_done = set()

    def begin_iteration(self, zero_grads=True):
        self.st.stage_begin_iteration()
        self.bwd_done = set()
        if zero_grads:
            self.st.zero_grads()
        if self.succ is not None:
            self.succ.stage_begin_iteration()
            self.succ_fwd_done = set()
            if zero_grads:
                self.succ.zero_grads()

    def _successor_backward(self, k):
        """What the live successor does between SEND_ACT(k) and RECV_GRAD(k)."""
        torch = self.st.torch
        succ = self.succ
        # the successor works on its own stream; order it after our forward
        succ.stream_main.wait_stream(self.st.stream_main)
        if k not in self.succ_fwd_done:
            succ.stage_fwd(k, self.y[k], self.z_succ[k])
            self.succ_fwd_done.add(k)
        succ.stage_bwd(k, self.gz[k], self.gy[k])
        self.st.stream_main.wait_stream(succ.stream_main)

    def _comm(self, op, lane, k, arg):
        """Hook for the communication instructions: the live successor's work happens where its
        gradient is received.  Nothing here ever reports a lost peer (the tests and the benchmark
        decide themselves when the successor is gone)."""
        if op == B.RECV_GRAD and arg == self.st.cfg.stage_id + 1 and self.succ is not None and not self.st.merged:
            self._successor_backward(k)
        return False

    def run(self, program):
        """The library interprets the list (stage_run); this side only supplies the buffer tables and,
        through the hook, the neighbours."""
        st = self.st
        # replayed BRCs (their own backward already ran) write their input gradient to buffers of their own
        done = set(self.bwd_done)
        replay = [None] * st.cfg.M
        for op, lane, k, arg in program:
            if op == B.BWD:
                done.add(k)
            elif op == B.BRC and st.merged and (k in done or st.cfg.data_parallel):
                self.gy_replay[k] = replay[k] = st.new_act()
        n = st.stage_run(program, x=self.x, y=self.y, frc_in=self.frc_in, z=self.z_frc, gy=self.gy, gx=self.gx,
                         gz=self.gz, gy_replay=replay if any(r is not None for r in replay) else None,
                         us_per_tick=self.us_per_tick, adam=self.adam,
                         comm=self._comm if self.succ is not None else None)
        assert n == len(program)
        self.bwd_done = done
        if self.adam is not None and any(op == B.APPLY for op, _, _, _ in program):
            # the stage has updated itself (APPLY inside stage_run); its live successor updates too, and the
            # replica then takes the successor's new parameters and optimizer state
            self.step += 1
            if self.succ is not None and not st.merged:
                self.succ.stage_apply(self.step, **self.adam)
                st.stream_main.wait_stream(self.succ.stream_main)
                st.stage_sync_replica(self.succ.own_w, self.succ.own_opt)
        return self

    def sync(self):
        self.st.stage_sync()
        if self.succ is not None:
            self.succ.stage_sync()


class WrapHarness:
    """Interpreter around the wrap-around stage: a Stage with cfg.wrap plus the model's Ends.  The stage
    before the last (P-2) is a table of inputs x_k, the samples are tables of token ids and labels, and the
    second stage, which returns the gradient at the first stage's output, is the table g1_k.  Every
    compute instruction is the pair of C ABI calls that the ends' header gives for it."""

    def __init__(self, stage, ends, x, ids, labels, g1, us_per_tick=0.0):
        torch = stage.torch
        self.st, self.ends = stage, ends
        self.x, self.ids, self.labels, self.g1 = x, ids, labels, g1
        self.us_per_tick = us_per_tick
        M = stage.cfg.M
        self.y = [stage.new_act() for _ in range(M)]
        self.gy = [stage.new_act() for _ in range(M)]
        self.gx = [stage.new_act() for _ in range(M)]
        self.x0 = [stage.new_act() for _ in range(M)]
        self.z_frc = [stage.new_act() for _ in range(M)]
        self.dx0 = [stage.new_act() for _ in range(M)]
        self.loss = torch.zeros(M, dtype=torch.float32, device=stage.device)

    def begin_iteration(self, zero_grads=True):
        self.st.stage_begin_iteration()
        self.ends.ends_begin_iteration()
        if zero_grads:
            self.st.zero_grads()
            self.ends.zero_grads(self.st.stream_main)

    def run(self, program):
        st, en = self.st, self.ends
        main = st.stream_main
        for op, lane, k, arg in program:
            if op == B.FWD:
                st.stage_fwd(k, self.x[k], self.y[k])
                en.ends_back_fwd(self.y[k], self.labels[k], self.loss[k:k + 1], main)
            elif op == B.BWD:
                en.ends_back_bwd(self.gy[k], main)
                st.stage_bwd(k, self.gy[k], self.gx[k])
            elif op == B.FRC:
                s_frc = main if st.merged else st.stream_frc
                en.ends_front_fwd(k, self.ids[k], self.x0[k], s_frc)
                st.shadow_fwd_frc(k, self.x0[k], self.z_frc[k])
            elif op == B.BRC:
                st.shadow_bwd_brc(k, self.g1[k], self.dx0[k])
                en.ends_front_bwd(k, self.dx0[k], main)
            elif op == B.BUBBLE:
                if self.us_per_tick > 0:
                    st.stage_bubble(arg, self.us_per_tick)
            elif op == B.JOIN:
                st.stage_join()
        return self

    def sync(self):
        self.st.stage_sync()


def split_at_failure(program, k_fail):
    """The instructions that ran before the failure was noticed: up to and
    including FWD(k_fail) and its FRC."""
    last = max(i for i, ins in enumerate(program) if ins[2] == k_fail and ins[0] in (B.FWD, B.FRC))
    return program[:last + 1]
