"""One Bamboo stage executing an instruction list (oracle; test infrastructure).

Section 5.1: node s runs normal computation (FNC/BNC) over its own layers and
redundant computation (FRC/BRC) over a replica of its successor's layers.
Section 5.2: FRC is eager and its intermediates are kept until a preemption;
BRC is lazy and recomputes the gradients lost with the victim.

Neighbours are simulated in the same process:
  stage s-1  = a table of inputs x_k
  stage s+1  = the same layer code over the shadow parameter values, with its own
               caches and its own gradient accumulator (lost on preemption)
  stage s+2  = a table of upstream gradients g_z_k
"""
import numpy as np

from . import layer as L
from . import schedule as S


def stash_record_index(slot, layer, n_layers):
    """Index of the record (slot, layer) inside a stash arena, in records."""
    return slot * n_layers + layer


def _acc(dst, grads):
    """dst += grads, layer by layer, tensor by tensor."""
    for d, g in zip(dst, grads):
        for name in L.PARAM_NAMES:
            d[name] = d[name] + g[name]


def _zeros_like_params(layers):
    return [{n: np.zeros_like(p[n]) for n in L.PARAM_NAMES} for p in layers]


class StageSim:
    def __init__(self, arch, own_layers, shadow_layers, B, S_len, n_h, P, s, M,
                 x_table, gz_table, eps=1e-5):
        self.arch, self.B, self.S, self.n_h, self.eps = arch, B, S_len, n_h, eps
        self.own, self.shadow = own_layers, shadow_layers
        self.P, self.s, self.M = P, s, M
        self.x, self.gz = x_table, gz_table
        self.C_own = S.own_slots(P, s, M)
        self.own_stash = {}        # slot -> (k, caches)
        self.shadow_stash = {}     # slot -> (k, caches)
        self.G_own = _zeros_like_params(own_layers)
        self.G_shadow = _zeros_like_params(shadow_layers)
        # simulated successor
        self.succ_alive = True
        self.succ_cache = {}
        self.G_succ = _zeros_like_params(shadow_layers)
        self.succ_bwd_done = []
        self.y, self.z_frc, self.z_succ, self.gy, self.gx = {}, {}, {}, {}, {}
        self.bwd_done = set()
        self.trace = []

    # ---- the successor's own work (only while it is alive)
    def _succ_backward(self, k):
        if k not in self.succ_cache:
            self.z_succ[k], self.succ_cache[k] = L.stack_fwd(
                self.arch, self.shadow, self.y[k], self.B, self.S, self.n_h, self.eps)
        gy, grads = L.stack_bwd(self.arch, self.shadow, self.succ_cache.pop(k), self.gz[k])
        _acc(self.G_succ, grads)
        self.succ_bwd_done.append(k)
        return gy

    def preempt_successor(self):
        """The successor disappears: its caches and accumulated gradients are gone."""
        self.succ_alive = False
        self.succ_cache = {}
        self.G_succ = None

    # ---- interpreter
    def run(self, prog):
        for op, lane, k, arg in prog:
            self.trace.append((op, k))
            if op == S.FWD:
                assert arg == k % self.C_own
                assert arg not in self.own_stash, "own stash slot %d still live" % arg
                self.y[k], caches = L.stack_fwd(self.arch, self.own, self.x[k],
                                                self.B, self.S, self.n_h, self.eps)
                self.own_stash[arg] = (k, caches)
            elif op == S.FRC:
                assert arg == k and k in self.y
                assert arg not in self.shadow_stash
                self.z_frc[k], caches = L.stack_fwd(self.arch, self.shadow, self.y[k],
                                                    self.B, self.S, self.n_h, self.eps)
                self.shadow_stash[arg] = (k, caches)
            elif op == S.RECV_GRAD:
                if arg == self.s + 1:          # from the live successor
                    assert self.succ_alive
                    self.gy[k] = self._succ_backward(k)
                # from s+2 (after failover): g_z_k is read from the table by BRC
            elif op == S.BWD:
                kk, caches = self.own_stash.pop(arg)
                assert kk == k
                self.gx[k], grads = L.stack_bwd(self.arch, self.own, caches, self.gy[k])
                _acc(self.G_own, grads)
                self.bwd_done.add(k)
            elif op == S.BRC:
                kk, caches = self.shadow_stash.pop(arg)
                assert kk == k
                gy, grads = L.stack_bwd(self.arch, self.shadow, caches, self.gz[k])
                _acc(self.G_shadow, grads)
                if k not in self.bwd_done:     # replayed micro-batches already have theirs
                    self.gy[k] = gy
                else:
                    self.gy_replay = getattr(self, "gy_replay", {})
                    self.gy_replay[k] = gy
            # SEND_*, RECV_ACT, BUBBLE, JOIN, ALLREDUCE, APPLY: no arithmetic
        return self


def run_no_failure(arch, own, shadow, B, S_len, n_h, P, s, M, x, gz, frc=True, eps=1e-5, rc=None):
    sim = StageSim(arch, own, shadow, B, S_len, n_h, P, s, M, x, gz, eps)
    return sim.run(S.stage_program(P, s, M, frc=frc, rc=rc))


def run_with_failure(arch, own, shadow, B, S_len, n_h, P, s, M, x, gz, k_fail, eps=1e-5, rc=S.EFLB):
    sim = StageSim(arch, own, shadow, B, S_len, n_h, P, s, M, x, gz, eps)
    sim.run(S.prefix_until_failure(P, s, M, k_fail, rc=rc))
    sim.preempt_successor()
    return sim.run(S.failover_program(P, s, M, k_fail, rc=rc))


# ---- wrap-around: the last stage holds the replica of the first (Section 5.1) ------------

class WrapStageSim:
    """The last stage (own layers + the model's back end: LM head and loss) shadowing the first
    stage (the model's front end: embedding, + its layers), which takes the samples' token ids
    as input -- the last node fetches them itself.  Backward of the own layers starts from the
    loss; BRC starts from the gradient the second stage sends (a table here)."""

    def __init__(self, arch, own_layers, back, shadow_layers, front, B, S_len, n_h, P, M,
                 x_table, labels, ids, g1_table, eps=1e-5):
        from . import ends as E
        self.E = E
        self.arch, self.B, self.S, self.n_h, self.eps = arch, B, S_len, n_h, eps
        self.own, self.back, self.shadow, self.front = own_layers, back, shadow_layers, front
        self.P, self.M = P, M
        self.x, self.labels, self.ids, self.g1 = x_table, labels, ids, g1_table
        self.C_own = S.own_slots(P, P - 1, M)
        self.own_stash, self.shadow_stash = {}, {}
        self.G_own = _zeros_like_params(own_layers)
        self.G_shadow = _zeros_like_params(shadow_layers)
        self.G_back = {n: np.zeros_like(v) for n, v in back.items()}
        self.G_front = {n: np.zeros_like(v) for n, v in front.items()}
        self.loss, self.z_frc, self.gx, self.dx0 = {}, {}, {}, {}

    def run(self, prog):
        E = self.E
        for op, lane, k, arg in prog:
            if op == S.FWD:
                assert arg == k % self.C_own and arg not in self.own_stash
                y, caches = L.stack_fwd(self.arch, self.own, self.x[k], self.B, self.S, self.n_h, self.eps)
                self.loss[k], _, cb = E.back_fwd(self.arch, self.back, y, self.labels[k], self.eps)
                self.own_stash[arg] = (k, caches, cb)
            elif op == S.BWD:
                kk, caches, cb = self.own_stash.pop(arg)
                assert kk == k
                dy, gb = E.back_bwd(self.arch, self.back, cb)
                self.gx[k], grads = L.stack_bwd(self.arch, self.own, caches, dy)
                _acc(self.G_own, grads)
                for n in gb:
                    self.G_back[n] = self.G_back[n] + gb[n]
            elif op == S.FRC:
                assert arg == k and k not in self.shadow_stash
                x0, cf = E.front_fwd(self.arch, self.front, self.ids[k], self.S, self.eps)
                self.z_frc[k], caches = L.stack_fwd(self.arch, self.shadow, x0, self.B, self.S, self.n_h, self.eps)
                self.shadow_stash[k] = (caches, cf)
            elif op == S.BRC:
                caches, cf = self.shadow_stash.pop(arg)
                self.dx0[k], grads = L.stack_bwd(self.arch, self.shadow, caches, self.g1[k])
                _acc(self.G_shadow, grads)
                gf = E.front_bwd(self.arch, self.front, cf, self.dx0[k])
                for n in gf:
                    self.G_front[n] = self.G_front[n] + gf[n]
        return self


def wrap_first_stage_reference(arch, layers, front, B, S_len, n_h, M, ids, g1_table, eps=1e-5):
    """What the first stage itself accumulates over an iteration without a failure: gradients of
    its layers and of the model's front end (what failover has to reproduce)."""
    from . import ends as E
    G = _zeros_like_params(layers)
    Gf = {n: np.zeros_like(v) for n, v in front.items()}
    z = {}
    for k in range(M):
        x0, cf = E.front_fwd(arch, front, ids[k], S_len, eps)
        z[k], caches = L.stack_fwd(arch, layers, x0, B, S_len, n_h, eps)
        dx0, grads = L.stack_bwd(arch, layers, caches, g1_table[k])
        _acc(G, grads)
        gf = E.front_bwd(arch, front, cf, dx0)
        for n in gf:
            Gf[n] = Gf[n] + gf[n]
    return G, Gf, z


# ---- pure data parallelism (Section 5.2, "Support for Pure Data Parallelism") ------------------

class DataParallelSim:
    """A node of a pure data-parallel job: it holds the whole model and, as redundancy, the replica of
    another node's parameters (and optimizer state).  There is no bubble; eager FRC means the node
    also runs the forward of the OTHER node's micro-batch k through the replica ("over-batching": its
    own minibatch plus a redundant one) and keeps the intermediates; lazy BRC back-propagates them,
    with the other node's upstream gradient, once that node is lost.

    own_layers / replica_layers: this node's and the other node's parameters (equal values in a
    synchronous job, kept as separate copies as the paper keeps them);
    x, g: this node's micro-batches and the gradients at its output (stand-ins for the loss);
    xn, gn: the same for the node whose replica is held.
    The other node is simulated until preempted: G_neigh accumulates what it computes itself."""

    def __init__(self, arch, own_layers, replica_layers, B, S_len, n_h, M, x, g, xn, gn, eps=1e-5):
        self.arch, self.B, self.S, self.n_h, self.eps = arch, B, S_len, n_h, eps
        self.own, self.shadow, self.M = own_layers, replica_layers, M
        self.x, self.g, self.xn, self.gn = x, g, xn, gn
        self.own_stash, self.shadow_stash = {}, {}
        self.G_own = _zeros_like_params(own_layers)
        self.G_shadow = _zeros_like_params(replica_layers)
        self.G_neigh = _zeros_like_params(replica_layers)
        self.y, self.z_frc, self.gx, self.gxn = {}, {}, {}, {}
        self.neigh_alive = True

    def _neighbour_step(self, k):
        """The other node's own forward + backward of its micro-batch k (while it lives)."""
        z, caches = L.stack_fwd(self.arch, self.shadow, self.xn[k], self.B, self.S, self.n_h, self.eps)
        _, grads = L.stack_bwd(self.arch, self.shadow, caches, self.gn[k])
        _acc(self.G_neigh, grads)
        return z

    def preempt_neighbour(self):
        self.neigh_alive = False
        self.G_neigh = None

    def run(self, prog):
        for op, lane, k, arg in prog:
            if op == S.FWD:
                assert arg == 0 and arg not in self.own_stash        # one slot: forward, then its backward
                self.y[k], caches = L.stack_fwd(self.arch, self.own, self.x[k], self.B, self.S, self.n_h, self.eps)
                self.own_stash[arg] = (k, caches)
            elif op == S.FRC:
                assert arg == k and k not in self.shadow_stash
                self.z_frc[k], caches = L.stack_fwd(self.arch, self.shadow, self.xn[k], self.B, self.S, self.n_h,
                                                    self.eps)
                self.shadow_stash[k] = caches
            elif op == S.BWD:
                kk, caches = self.own_stash.pop(arg)
                assert kk == k
                self.gx[k], grads = L.stack_bwd(self.arch, self.own, caches, self.g[k])
                _acc(self.G_own, grads)
            elif op == S.BRC:
                self.gxn[k], grads = L.stack_bwd(self.arch, self.shadow, self.shadow_stash.pop(arg), self.gn[k])
                _acc(self.G_shadow, grads)
        return self
