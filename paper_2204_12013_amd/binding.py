"""Thin ctypes binding over libbamboo_stage.so (argument marshalling only).

Every step of the hot path runs inside the library's HIP kernels.  PyTorch is
used for device memory and streams.  There is no fallback: if the native
library has not been built, importing this module raises.
"""
import ctypes as C
import os

import numpy as np
# torch ships its own HIP runtime; it has to be in the process before the
# library is loaded so that both resolve to the same runtime (two runtimes in
# one process cannot share streams or memory)
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbamboo_stage.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("native library missing: %s (build it with `python %s`)"
                      % (LIB_PATH, os.path.join(_HERE, "build.py")))
lib = C.CDLL(LIB_PATH)

OK, E_BADCFG, E_BADMB, E_STATE, E_HIP, E_ARG, E_NOMEM = 0, -1, -2, -3, -4, -5, -6
(RECV_ACT, SEND_ACT, RECV_GRAD, SEND_GRAD, FWD, BWD, FRC, BRC, BUBBLE, JOIN, ALLREDUCE, APPLY) = range(12)
# launch sites of the per-site timing (enum bamboo_kernel_class in bamboo_debug.h)
KERNEL_CLASSES = ("gemm_qkv", "gemm_attn_out", "gemm_ffn1", "gemm_ffn2", "dgrad_ffn2", "dgrad_ffn1", "dgrad_attn_out",
                  "dgrad_qkv", "wgrad_group", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd", "colsum")


class Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("arch", "dtype", "hidden", "heads", "ffn", "seq", "micro_batch", "n_own", "n_shadow",
                 "P", "stage_id", "M", "rc_mode", "tick_F", "tick_B")] + [("ln_eps", C.c_float), ("swap_slots", C.c_int32), ("wrap", C.c_int32),
                                                                        ("data_parallel", C.c_int32)]


class Instr(C.Structure):
    _fields_ = [("op", C.c_uint8), ("lane", C.c_uint8), ("mb", C.c_int16), ("arg", C.c_int32)]


class Sizes(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in
                ("own_w", "shadow_w", "own_g", "shadow_g", "own_stash", "shadow_stash", "workspace",
                 "rec_bytes", "layer_params")] + [("c_own", C.c_int32), ("c_shadow", C.c_int32)] + \
        [("own_opt", C.c_uint64), ("shadow_opt", C.c_uint64), ("host_stash", C.c_uint64)]


class EndsSizes(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in
                ("front_params", "back_params", "front_w", "back_w", "front_g", "back_g", "front_stash",
                 "back_stash", "workspace")]


class Adam(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float)]


COMM_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.POINTER(Instr))


class Tables(C.Structure):
    """bamboo_tables_t: per-micro-batch buffer tables and the hooks of stage_run."""
    _fields_ = [("x", C.POINTER(C.c_void_p)), ("y", C.POINTER(C.c_void_p)), ("frc_in", C.POINTER(C.c_void_p)),
                ("z", C.POINTER(C.c_void_p)), ("gy", C.POINTER(C.c_void_p)), ("gx", C.POINTER(C.c_void_p)),
                ("gz", C.POINTER(C.c_void_p)), ("gy_replay", C.POINTER(C.c_void_p)), ("us_per_tick", C.c_float),
                ("adam", C.POINTER(Adam)), ("comm", COMM_FN), ("user", C.c_void_p)]


class BambooError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, lib.stage_strerror(status).decode(), status))


_vp, _i32, _i64, _f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
_cfgp, _insp, _szp = C.POINTER(Cfg), C.POINTER(Instr), C.POINTER(Sizes)
_SIGS = {
    "stage_query_sizes": (C.c_int, [_cfgp, _szp]),
    "stage_program": (C.c_int, [_cfgp, _insp, _i32]),
    "stage_program_uneven": (C.c_int, [_cfgp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), _insp, _i32]),
    "stage_failover_program": (C.c_int, [_cfgp, _i32, _insp, _i32]),
    "stage_merged_program": (C.c_int, [_cfgp, _insp, _i32]),
    "stage_run": (C.c_int, [_vp, _insp, _i32, C.POINTER(Tables)]),
    "stage_wrap_victim_progress": (C.c_int, [_cfgp, _i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "stage_record_offset": (_i64, [_cfgp, _i32, _i32, _i32]),
    "stage_strerror": (C.c_char_p, [C.c_int]),
    "stage_record_fields": (C.c_int, [_cfgp, C.POINTER(C.c_uint64)]),
    "stage_workspace_fields": (C.c_int, [_cfgp, C.POINTER(C.c_uint64)]),
    "stage_init": (C.c_int, [_cfgp, _szp] + [_vp] * 9 + [C.POINTER(_vp)]),
    "stage_schedule": (C.c_int, [_vp, _insp, _i32]),
    "stage_begin_iteration": (C.c_int, [_vp]),
    "stage_fwd": (C.c_int, [_vp, _i32, _vp, _vp]),
    "shadow_fwd_frc": (C.c_int, [_vp, _i32, _vp, _vp]),
    "stage_bwd": (C.c_int, [_vp, _i32, _vp, _vp]),
    "shadow_bwd_brc": (C.c_int, [_vp, _i32, _vp, _vp]),
    "failover_merge": (C.c_int, [_vp, _i32, _insp, _i32]),
    "stage_bubble": (C.c_int, [_vp, _i32, _f32]),
    "stage_optimizer_init": (C.c_int, [_vp, _vp, _vp]),
    "stage_apply": (C.c_int, [_vp, C.POINTER(Adam), _i32]),
    "stage_sync_replica": (C.c_int, [_vp, _vp, _vp]),
    "stage_swap_attach": (C.c_int, [_vp, _vp, C.c_uint64, _vp]),
    "stage_join": (C.c_int, [_vp]),
    "stage_sync": (C.c_int, [_vp]),
    "stage_destroy": (C.c_int, [_vp]),
    "stage_profile": (C.c_int, [_vp, C.c_int]),
    "stage_profile_read": (C.c_int, [_vp, _i32, C.POINTER(C.c_double), C.POINTER(_i64), C.POINTER(C.c_double)]),
    "ends_query_sizes": (C.c_int, [_cfgp, _i32, C.POINTER(EndsSizes)]),
    "ends_init": (C.c_int, [_cfgp, _i32, C.POINTER(EndsSizes)] + [_vp] * 7 + [C.POINTER(_vp)]),
    "ends_front_fwd": (C.c_int, [_vp, _i32, _vp, _vp, _vp]),
    "ends_front_bwd": (C.c_int, [_vp, _i32, _vp, _vp]),
    "ends_back_fwd": (C.c_int, [_vp, _vp, _vp, _vp, _vp]),
    "ends_back_bwd": (C.c_int, [_vp, _vp, _vp]),
    "ends_begin_iteration": (C.c_int, [_vp]),
    "ends_destroy": (C.c_int, [_vp]),
    "bk_linear_fwd": (C.c_int, [C.c_int] * 5 + [_vp] * 7),
    "bk_linear_bwd_input": (C.c_int, [C.c_int] * 5 + [_vp] * 6),
    "bk_linear_bwd_weight": (C.c_int, [C.c_int] * 5 + [_vp] * 6),
    "bk_linear_bwd_weight_group": (C.c_int, [C.c_int, C.c_int] + [C.POINTER(C.c_int)] * 3 + [C.POINTER(_vp)] * 3 + [_vp]),
    "bk_colsum_acc": (C.c_int, [C.c_int] * 3 + [_vp] * 4),
    "bk_colsum_scratch_floats": (C.c_uint64, [C.c_int]),
    "bk_colsum_acc_static": (C.c_int, [C.c_int] * 3 + [_vp] * 3),
    "bk_colsum_static_max_floats": (C.c_uint64, []),
    "bk_attention_fwd": (C.c_int, [C.c_int] * 7 + [_vp] * 4),
    "bk_attention_bwd": (C.c_int, [C.c_int] * 7 + [_vp] * 7),
    "bk_layernorm_fwd": (C.c_int, [C.c_int] * 3 + [_f32] + [_vp] * 6),
    "bk_layernorm_bwd": (C.c_int, [C.c_int] * 3 + [_vp] * 10),
    "bk_layernorm_bwd_scratch_floats": (C.c_uint64, [C.c_int]),
    "bk_copy": (C.c_int, [_vp, _vp, C.c_uint64, _vp]),
    "bk_embedding_fwd": (C.c_int, [C.c_int] * 5 + [_vp] * 5),
    "bk_embedding_bwd": (C.c_int, [C.c_int] * 5 + [_vp] * 5),
    "bk_softmax_xent_fwd": (C.c_int, [C.c_int] * 3 + [_vp] * 5),
    "bk_softmax_xent_bwd": (C.c_int, [C.c_int] * 3 + [_vp] * 3 + [C.c_float, _vp, _vp]),
    "bk_ordered_sum": (C.c_int, [C.c_int64, _vp, C.c_float, _vp, _vp]),
    "bk_gemm_tile": (C.c_int, [C.c_int]),
    "bk_gemm_stages": (C.c_int, [C.c_int]),
    "bk_adam": (C.c_int, [C.c_int, C.c_int64] + [_vp] * 5 + [C.c_float] * 4 + [C.c_int, _vp]),
}
EXPORTS = tuple(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args


def _check(status, where):
    if status < 0:
        raise BambooError(status, where)
    return status


RC_LFLB, RC_EFLB, RC_EFEB = 0, 1, 2


def make_cfg(sc, frc_enabled=True, tick_F=1, tick_B=2, ln_eps=1e-5, rc_mode=None, **override):
    """rc_mode (RC_LFLB / RC_EFLB / RC_EFEB) overrides frc_enabled (True = EFLB, False = LFLB)."""
    if rc_mode is None:
        rc_mode = RC_EFLB if frc_enabled else RC_LFLB
    """Cfg from a synth.StageConfig (or anything with the same attributes)."""
    vals = dict(arch=sc.arch, dtype=sc.dtype, hidden=sc.hidden, heads=sc.heads, ffn=sc.ffn, seq=sc.seq,
                micro_batch=sc.micro_batch, n_own=sc.n_own, n_shadow=sc.n_shadow, P=sc.P,
                stage_id=sc.stage_id, M=sc.M, rc_mode=int(rc_mode), tick_F=tick_F, tick_B=tick_B,
                ln_eps=ln_eps, swap_slots=0, wrap=0, data_parallel=0)
    vals.update(override)
    return Cfg(**vals)


def _instr_list(arr, n):
    return [(int(i.op), int(i.lane), int(i.mb), int(i.arg)) for i in arr[:n]]


def stage_wrap_victim_progress(cfg, k_fail):
    a, b = C.c_int32(), C.c_int32()
    _check(lib.stage_wrap_victim_progress(C.byref(cfg), k_fail, C.byref(a), C.byref(b)), "stage_wrap_victim_progress")
    return a.value, b.value


def stage_query_sizes(cfg):
    sz = Sizes()
    _check(lib.stage_query_sizes(C.byref(cfg), C.byref(sz)), "stage_query_sizes")
    return sz


def stage_program(cfg):
    n = _check(lib.stage_program(C.byref(cfg), None, 0), "stage_program")
    arr = (Instr * n)()
    _check(lib.stage_program(C.byref(cfg), arr, n), "stage_program")
    return _instr_list(arr, n)


def stage_program_uneven(cfg, tick_F=None, tick_B=None):
    """stage_program with a forward / backward duration per stage (sequences of P ints or None)."""
    def arr_of(t):
        return None if t is None else (C.c_int32 * cfg.P)(*[int(v) for v in t])
    f, b = arr_of(tick_F), arr_of(tick_B)
    n = _check(lib.stage_program_uneven(C.byref(cfg), f, b, None, 0), "stage_program_uneven")
    arr = (Instr * n)()
    _check(lib.stage_program_uneven(C.byref(cfg), f, b, arr, n), "stage_program_uneven")
    return _instr_list(arr, n)


def stage_failover_program(cfg, k_fail):
    n = _check(lib.stage_failover_program(C.byref(cfg), k_fail, None, 0), "stage_failover_program")
    arr = (Instr * n)()
    _check(lib.stage_failover_program(C.byref(cfg), k_fail, arr, n), "stage_failover_program")
    return _instr_list(arr, n)


def stage_merged_program(cfg):
    n = _check(lib.stage_merged_program(C.byref(cfg), None, 0), "stage_merged_program")
    arr = (Instr * n)()
    _check(lib.stage_merged_program(C.byref(cfg), arr, n), "stage_merged_program")
    return _instr_list(arr, n)


def pointer_table(tensors):
    """A C array of the device addresses of a list of tensors (None entries become NULL), or None."""
    if tensors is None:
        return None
    return (C.c_void_p * len(tensors))(*[None if t is None else t.data_ptr() for t in tensors])


def instr_array(program):
    arr = (Instr * max(len(program), 1))()
    for i, (op, lane, mb, arg) in enumerate(program):
        arr[i].op, arr[i].lane, arr[i].mb, arr[i].arg = op, lane, mb, arg
    return arr


def stage_record_offset(cfg, kind, slot, layer):
    return _check(lib.stage_record_offset(C.byref(cfg), kind, slot, layer), "stage_record_offset")


RECORD_FIELDS = ("x", "ain", "qkv", "ctx", "r1", "fin", "g", "dg", "r2", "lse", "ln1", "ln2", "rec_bytes")


def stage_record_fields(cfg):
    arr = (C.c_uint64 * 13)()
    _check(lib.stage_record_fields(C.byref(cfg), arr), "stage_record_fields")
    return dict(zip(RECORD_FIELDS, [int(v) for v in arr]))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


WORKSPACE_FIELDS = ("dh", "d1", "d2", "d3", "dctx", "dqkv", "bytes")


def stage_workspace_fields(cfg):
    arr = (C.c_uint64 * 7)()
    _check(lib.stage_workspace_fields(C.byref(cfg), arr), "stage_workspace_fields")
    return dict(zip(WORKSPACE_FIELDS, [int(v) for v in arr]))


class Stage:
    """Owns the device buffers (as torch tensors) and the two streams of one
    stage and forwards every call to the C ABI."""

    def __init__(self, cfg, own_w, shadow_w, device="cuda:0", attach_swap=True):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        self.sizes = sz = stage_query_sizes(cfg)
        self.act_dtype = torch.bfloat16 if cfg.dtype == 1 else torch.float32
        self.T, self.H = cfg.micro_batch * cfg.seq, cfg.hidden

        def buf(nbytes):
            return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=self.device)
        assert own_w.dtype == self.act_dtype and own_w.numel() == sz.layer_params * cfg.n_own
        self.own_w = own_w.to(self.device).contiguous()
        self.shadow_w = None
        if cfg.n_shadow > 0:
            assert shadow_w.dtype == self.act_dtype and shadow_w.numel() == sz.layer_params * cfg.n_shadow
            self.shadow_w = shadow_w.to(self.device).contiguous()
        self.own_g = torch.zeros(int(sz.layer_params) * cfg.n_own, dtype=torch.float32, device=self.device)
        self.shadow_g = torch.zeros(max(int(sz.layer_params) * cfg.n_shadow, 1), dtype=torch.float32,
                                    device=self.device)
        self.own_stash = buf(sz.own_stash)
        self.shadow_stash = buf(sz.shadow_stash)
        self.workspace = buf(sz.workspace)
        self.stream_main = torch.cuda.Stream(device=self.device)
        self.stream_frc = torch.cuda.Stream(device=self.device)
        self._h = C.c_void_p()
        self._shadow_g_dirty = False       # shadow_g starts as zeros
        self.merged = False
        self.own_opt = self.shadow_opt = None
        torch.cuda.synchronize(self.device)
        _check(lib.stage_init(C.byref(cfg), C.byref(sz), _ptr(self.own_w), _ptr(self.shadow_w), _ptr(self.own_g),
                              _ptr(self.shadow_g) if cfg.n_shadow > 0 else None, _ptr(self.own_stash),
                              _ptr(self.shadow_stash) if cfg.n_shadow > 0 else None, _ptr(self.workspace),
                              C.c_void_p(self.stream_main.cuda_stream), C.c_void_p(self.stream_frc.cuda_stream),
                              C.byref(self._h)), "stage_init")
        self.host_stash = self.stream_swap = None
        if cfg.swap_slots > 0 and attach_swap:
            # FRC results swapped out to the host: pinned memory allocated as such, a third stream
            self.host_stash = torch.empty(int(sz.host_stash), dtype=torch.uint8, pin_memory=True)
            self.stream_swap = torch.cuda.Stream(device=self.device)
            _check(lib.stage_swap_attach(self._h, C.c_void_p(self.host_stash.data_ptr()), int(sz.host_stash),
                                         C.c_void_p(self.stream_swap.cuda_stream)), "stage_swap_attach")

    def stash_tensor(self, kind, slot, layer, field):
        """View of one tensor of a stash record (kind 0 own, 1 shadow)."""
        torch = self.torch
        cfg = self.cfg
        f = stage_record_fields(cfg)
        base = stage_record_offset(cfg, kind, slot, layer) + f[field]
        arena = self.own_stash if kind == 0 else self.shadow_stash
        T, H, F = self.T, cfg.hidden, cfg.ffn
        es = 2 if cfg.dtype == 1 else 4
        if field in ("lse", "ln1", "ln2"):
            n = cfg.micro_batch * cfg.heads * cfg.seq if field == "lse" else 2 * T
            return arena[base:base + 4 * n].view(torch.float32)
        cols = {"qkv": 3 * H, "g": F, "dg": F}.get(field, H)
        return arena[base:base + es * T * cols].view(self.act_dtype).view(T, cols)

    def workspace_tensor(self, field):
        """View of one of lane 0's backward buffers (inspection after a backward pass has finished)."""
        cfg = self.cfg
        base = stage_workspace_fields(cfg)[field]
        es = 2 if cfg.dtype == 1 else 4
        cols = {"dh": cfg.ffn, "dqkv": 3 * cfg.hidden}.get(field, cfg.hidden)
        return self.workspace[base:base + es * self.T * cols].view(self.act_dtype).view(self.T, cols)

    def new_act(self):
        return self.torch.empty(self.T, self.H, dtype=self.act_dtype, device=self.device)

    def zero_grads(self):
        """Zeroes the gradient buffers on the main stream.  The replica's gradients are only ever written
        by BRC, so they are cleared only after one has run (a failure-free iteration leaves them zero)."""
        with self.torch.cuda.stream(self.stream_main):
            self.own_g.zero_()
            if self._shadow_g_dirty:
                self.shadow_g.zero_()
                self._shadow_g_dirty = False

    def stage_schedule(self):
        n = _check(lib.stage_schedule(self._h, None, 0), "stage_schedule")
        arr = (Instr * n)()
        _check(lib.stage_schedule(self._h, arr, n), "stage_schedule")
        return _instr_list(arr, n)

    def stage_begin_iteration(self):
        _check(lib.stage_begin_iteration(self._h), "stage_begin_iteration")

    def stage_fwd(self, k, x, y):
        _check(lib.stage_fwd(self._h, k, _ptr(x), _ptr(y)), "stage_fwd")

    def shadow_fwd_frc(self, k, y, z=None):
        _check(lib.shadow_fwd_frc(self._h, k, _ptr(y), _ptr(z)), "shadow_fwd_frc")

    def stage_bwd(self, k, gy, gx):
        _check(lib.stage_bwd(self._h, k, _ptr(gy), _ptr(gx)), "stage_bwd")

    def shadow_bwd_brc(self, k, gz, gy=None):
        self._shadow_g_dirty = True
        _check(lib.shadow_bwd_brc(self._h, k, _ptr(gz), _ptr(gy)), "shadow_bwd_brc")

    def failover_merge(self, k_fail):
        cap = 16 * self.cfg.M + 32
        arr = (Instr * cap)()
        n = _check(lib.failover_merge(self._h, k_fail, arr, cap), "failover_merge")
        self.merged = True
        return _instr_list(arr, n)

    def stage_run(self, program, x=None, y=None, frc_in=None, z=None, gy=None, gx=None, gz=None, gy_replay=None,
                  us_per_tick=0.0, adam=None, comm=None):
        """Hands an instruction list and the per-micro-batch buffer tables to the library's interpreter.
        comm(op, lane, mb, arg) -> bool is called for every communication instruction; a true return
        means the peer is gone.  Returns the number of instructions issued (len(program) unless comm
        stopped the run)."""
        keep = [pointer_table(v) for v in (x, y, frc_in, z, gy, gx, gz, gy_replay)]
        cast = lambda a: C.cast(a, C.POINTER(C.c_void_p)) if a is not None else None
        hp = Adam(**adam) if adam is not None else None
        failure = []

        def hook(user, ins):
            try:
                i = ins.contents
                return 1 if comm(int(i.op), int(i.lane), int(i.mb), int(i.arg)) else 0
            except BaseException as e:     # nothing may propagate through the C frames
                failure.append(e)
                return 1
        cb = COMM_FN(hook) if comm is not None else C.cast(None, COMM_FN)
        t = Tables(*[cast(a) for a in keep], us_per_tick, C.pointer(hp) if hp is not None else None, cb, None)
        arr = instr_array(program)
        n = lib.stage_run(self._h, arr, len(program), C.byref(t))
        if failure:
            raise failure[0]
        if any(op == BRC for op, _, _, _ in program[:max(n, 0)]):
            self._shadow_g_dirty = True
        return _check(n, "stage_run")

    def stage_optimizer_init(self):
        """Allocates the optimizer state ([master | m | v] fp32 for own and replica parameters)
        and has the library initialise it from the current parameters."""
        torch = self.torch
        self.own_opt = torch.empty(int(self.sizes.own_opt) // 4, dtype=torch.float32, device=self.device)
        self.shadow_opt = None
        if self.cfg.n_shadow > 0:
            self.shadow_opt = torch.empty(int(self.sizes.shadow_opt) // 4, dtype=torch.float32, device=self.device)
        torch.cuda.synchronize(self.device)
        _check(lib.stage_optimizer_init(self._h, _ptr(self.own_opt), _ptr(self.shadow_opt)), "stage_optimizer_init")

    def stage_apply(self, step, lr=6e-3, beta1=0.9, beta2=0.999, eps=1e-8):
        hp = Adam(lr, beta1, beta2, eps)
        _check(lib.stage_apply(self._h, C.byref(hp), step), "stage_apply")

    def stage_sync_replica(self, successor_w, successor_opt=None):
        _check(lib.stage_sync_replica(self._h, _ptr(successor_w), _ptr(successor_opt)), "stage_sync_replica")

    def stage_bubble(self, ticks, us_per_tick):
        _check(lib.stage_bubble(self._h, ticks, us_per_tick), "stage_bubble")

    def stage_join(self):
        _check(lib.stage_join(self._h), "stage_join")

    def stage_sync(self):
        _check(lib.stage_sync(self._h), "stage_sync")

    def stage_profile(self, enable):
        _check(lib.stage_profile(self._h, int(enable)), "stage_profile")

    def stage_profile_read(self, kernel_class):
        """(total ms, launches, algorithmic work) of one kernel class."""
        ms, n, w = C.c_double(), C.c_int64(), C.c_double()
        _check(lib.stage_profile_read(self._h, kernel_class, C.byref(ms), C.byref(n), C.byref(w)),
               "stage_profile_read")
        return ms.value, n.value, w.value

    def stage_destroy(self):
        if self._h:
            lib.stage_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.stage_destroy()
        except Exception:
            pass


# ---- individual kernels (tensors are torch device tensors) -------------------

def _stream(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _dt(t):
    import torch
    return 1 if t.dtype == torch.bfloat16 else 0


def bk_linear_fwd(X, W, bias, Y, res=None, gelu_out=None, impl=0, stream=None):
    T, K = X.shape
    N = W.shape[1]
    _check(lib.bk_linear_fwd(_dt(X), impl, T, N, K, _ptr(X), _ptr(W), _ptr(bias), _ptr(res), _ptr(Y),
                             _ptr(gelu_out), _stream(stream)), "bk_linear_fwd")


def bk_linear_bwd_input(dY, W, dX, res=None, mul=None, impl=0, stream=None):
    T, N = dY.shape
    K = W.shape[0]
    _check(lib.bk_linear_bwd_input(_dt(dY), impl, T, K, N, _ptr(dY), _ptr(W), _ptr(res), _ptr(mul), _ptr(dX),
                                   _stream(stream)), "bk_linear_bwd_input")


def bk_linear_bwd_weight(X, dY, dW, db=None, impl=0, stream=None):
    import torch
    T, K = X.shape
    N = dY.shape[1]
    partial = None
    if db is not None:
        partial = torch.empty(int(lib.bk_colsum_scratch_floats(N)), dtype=torch.float32, device=X.device)
    _check(lib.bk_linear_bwd_weight(_dt(X), impl, T, K, N, _ptr(X), _ptr(dY), _ptr(dW), _ptr(db), _ptr(partial),
                                    _stream(stream)), "bk_linear_bwd_weight")
    return partial


def bk_linear_bwd_weight_group(Xs, dYs, dWs, stream=None):
    """dWs[i] += Xs[i]^T dYs[i] for up to four independent problems, as one launch where possible."""
    n = len(Xs)
    ints = lambda v: (C.c_int * n)(*v)
    ptrs = lambda ts: (_vp * n)(*[t.data_ptr() for t in ts])
    _check(lib.bk_linear_bwd_weight_group(_dt(Xs[0]), n, ints([x.shape[0] for x in Xs]), ints([x.shape[1] for x in Xs]),
                                          ints([y.shape[1] for y in dYs]), ptrs(Xs), ptrs(dYs), ptrs(dWs),
                                          _stream(stream)), "bk_linear_bwd_weight_group")


def bk_colsum_acc(A, out, stream=None):
    import torch
    T, N = A.shape
    partial = torch.empty(int(lib.bk_colsum_scratch_floats(N)), dtype=torch.float32, device=A.device)
    _check(lib.bk_colsum_acc(_dt(A), T, N, _ptr(A), _ptr(out), _ptr(partial), _stream(stream)), "bk_colsum_acc")
    return partial


def bk_colsum_acc_static(A, out, stream=None):
    """bk_colsum_acc without any allocation: the partial rows live inside the library."""
    T, N = A.shape
    _check(lib.bk_colsum_acc_static(_dt(A), T, N, _ptr(A), _ptr(out), _stream(stream)), "bk_colsum_acc_static")


def bk_attention_fwd(qkv, ctx, lse, batch, seq, heads, causal, impl=0, stream=None):
    d = qkv.shape[1] // 3 // heads
    _check(lib.bk_attention_fwd(_dt(qkv), impl, batch, seq, heads, d, int(causal), _ptr(qkv), _ptr(ctx), _ptr(lse),
                                _stream(stream)), "bk_attention_fwd")


def bk_attention_bwd(qkv, ctx, lse, dctx, dqkv, batch, seq, heads, causal, impl=0, stream=None):
    import torch
    d = qkv.shape[1] // 3 // heads
    delta = torch.empty(batch * heads * seq, dtype=torch.float32, device=qkv.device)
    _check(lib.bk_attention_bwd(_dt(qkv), impl, batch, seq, heads, d, int(causal), _ptr(qkv), _ptr(ctx), _ptr(lse),
                                _ptr(dctx), _ptr(dqkv), _ptr(delta), _stream(stream)), "bk_attention_bwd")
    return delta


def bk_layernorm_fwd(r, gamma, beta, y, stats, eps=1e-5, stream=None):
    T, H = r.shape
    _check(lib.bk_layernorm_fwd(_dt(r), T, H, eps, _ptr(r), _ptr(gamma), _ptr(beta), _ptr(y), _ptr(stats),
                                _stream(stream)), "bk_layernorm_fwd")


def bk_layernorm_bwd(dout, r, stats, gamma, dr, dgamma, dbeta, add=None, stream=None):
    import torch
    T, H = r.shape
    partial = torch.empty(int(lib.bk_layernorm_bwd_scratch_floats(H)), dtype=torch.float32, device=r.device)
    _check(lib.bk_layernorm_bwd(_dt(r), T, H, _ptr(dout), _ptr(r), _ptr(stats), _ptr(gamma), _ptr(add), _ptr(dr),
                                _ptr(dgamma), _ptr(dbeta), _ptr(partial), _stream(stream)), "bk_layernorm_bwd")
    return partial


def bk_copy(src, dst, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(lib.bk_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "bk_copy")


def bk_gemm_tile(code):
    """Force the MFMA GEMM output tile (10*WM + WN; 0 = automatic); returns the previous code."""
    return _check(lib.bk_gemm_tile(code), "bk_gemm_tile")


def bk_adam(g, master, m, v, w, step, lr=6e-3, beta1=0.9, beta2=0.999, eps=1e-8, stream=None):
    """One Adam step on flat tensors: fp32 g, master, m, v; w = storage-dtype copy of the new master."""
    _check(lib.bk_adam(_dt(w), master.numel(), _ptr(g), _ptr(master), _ptr(m), _ptr(v), _ptr(w), lr, beta1, beta2,
                       eps, step, _stream(stream)), "bk_adam")


def bk_embedding_fwd(ids, E_tok, E_pos, out, stream=None):
    """out[t] = E_tok[ids[t]] + E_pos[t mod seq]; ids int32 [T]."""
    V, H = E_tok.shape
    _check(lib.bk_embedding_fwd(_dt(E_tok), ids.numel(), E_pos.shape[0], H, V, _ptr(ids), _ptr(E_tok), _ptr(E_pos),
                                _ptr(out), _stream(stream)), "bk_embedding_fwd")


def bk_embedding_bwd(ids, g, dE_tok, dE_pos, stream=None):
    V, H = dE_tok.shape
    _check(lib.bk_embedding_bwd(_dt(g), ids.numel(), dE_pos.shape[0], H, V, _ptr(ids), _ptr(g), _ptr(dE_tok),
                                _ptr(dE_pos), _stream(stream)), "bk_embedding_bwd")


def bk_softmax_xent_fwd(logits, labels, lse, loss_tok, stream=None):
    T, V = logits.shape
    _check(lib.bk_softmax_xent_fwd(_dt(logits), T, V, _ptr(logits), _ptr(labels), _ptr(lse), _ptr(loss_tok),
                                   _stream(stream)), "bk_softmax_xent_fwd")


def bk_softmax_xent_bwd(logits, labels, lse, scale, dlogits, stream=None):
    T, V = logits.shape
    _check(lib.bk_softmax_xent_bwd(_dt(logits), T, V, _ptr(logits), _ptr(labels), _ptr(lse), float(scale),
                                   _ptr(dlogits), _stream(stream)), "bk_softmax_xent_bwd")


def bk_ordered_sum(x, scale, out, stream=None):
    _check(lib.bk_ordered_sum(x.numel(), _ptr(x), float(scale), _ptr(out), _stream(stream)), "bk_ordered_sum")


def bk_gemm_stages(n):
    """Force the LDS ring depth of the pipelined MFMA GEMM (2..4; 0 = automatic); returns the previous value."""
    return _check(lib.bk_gemm_stages(n), "bk_gemm_stages")


def ends_query_sizes(cfg, vocab):
    sz = EndsSizes()
    _check(lib.ends_query_sizes(C.byref(cfg), vocab, C.byref(sz)), "ends_query_sizes")
    return sz


class Ends:
    """The model's front (embedding) and back (LM head + loss) around a wrap-around stage: owns their
    device buffers and forwards every call to the C ABI."""

    def __init__(self, cfg, vocab, front_w, back_w, device="cuda:0"):
        import torch
        self.torch, self.cfg, self.vocab = torch, cfg, vocab
        self.device = torch.device(device)
        self.sizes = sz = ends_query_sizes(cfg, vocab)
        act = torch.bfloat16 if cfg.dtype == 1 else torch.float32
        assert front_w.dtype == act and front_w.numel() == sz.front_params
        assert back_w.dtype == act and back_w.numel() == sz.back_params
        self.front_w, self.back_w = front_w.to(self.device).contiguous(), back_w.to(self.device).contiguous()
        self.front_g = torch.zeros(int(sz.front_params), dtype=torch.float32, device=self.device)
        self.back_g = torch.zeros(int(sz.back_params), dtype=torch.float32, device=self.device)
        buf = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device=self.device)
        self.front_stash, self.back_stash, self.workspace = buf(sz.front_stash), buf(sz.back_stash), buf(sz.workspace)
        self._front_g_dirty = False        # front_g starts as zeros
        self._h = C.c_void_p()
        torch.cuda.synchronize(self.device)
        _check(lib.ends_init(C.byref(cfg), vocab, C.byref(sz), _ptr(self.front_w), _ptr(self.front_g),
                             _ptr(self.back_w), _ptr(self.back_g), _ptr(self.front_stash), _ptr(self.back_stash),
                             _ptr(self.workspace), C.byref(self._h)), "ends_init")

    def zero_grads(self, stream):
        with self.torch.cuda.stream(stream):
            if self._front_g_dirty:        # written by the front's backward (BRC) only
                self.front_g.zero_()
                self._front_g_dirty = False
            self.back_g.zero_()

    def ends_begin_iteration(self):
        _check(lib.ends_begin_iteration(self._h), "ends_begin_iteration")

    def ends_front_fwd(self, k, ids, x0, stream):
        _check(lib.ends_front_fwd(self._h, k, _ptr(ids), _ptr(x0), _stream(stream)), "ends_front_fwd")

    def ends_front_bwd(self, k, dx0, stream):
        self._front_g_dirty = True
        _check(lib.ends_front_bwd(self._h, k, _ptr(dx0), _stream(stream)), "ends_front_bwd")

    def ends_back_fwd(self, y, labels, loss, stream):
        _check(lib.ends_back_fwd(self._h, _ptr(y), _ptr(labels), _ptr(loss), _stream(stream)), "ends_back_fwd")

    def ends_back_bwd(self, gy, stream):
        _check(lib.ends_back_bwd(self._h, _ptr(gy), _stream(stream)), "ends_back_bwd")

    def ends_destroy(self):
        if self._h:
            _check(lib.ends_destroy(self._h), "ends_destroy")
            self._h = C.c_void_p()


# ---- numpy <-> device helpers (storage conversion only) ------------------------

def to_device(a_f32, dtype, device="cuda:0"):
    """float32 numpy array (already representable in the storage type) -> tensor."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a_f32, dtype=np.float32))
    return t.to(torch.bfloat16 if dtype == 1 else torch.float32).to(device)


def to_host(t):
    return t.detach().to("cpu").float().numpy().astype(np.float64)
