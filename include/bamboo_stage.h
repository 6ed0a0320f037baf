/*
 * bamboo_stage.h -- C ABI of the Bamboo stage hot path on MI355X (gfx950).
 *
 * One pipeline stage's per-micro-batch training computation with redundant
 * computation (arXiv 2204.12013, Section 5):
 *   FNC/BNC  forward/backward normal computation over the stage's own layers,
 *   FRC      eager forward redundant computation over a replica of the
 *            successor's layers (Section 5.1), issued on a second stream so that
 *            it falls into the pipeline bubble or overlaps the next forward
 *            (Section 5.2 "Eager FRC", "Scheduling"),
 *   BRC      lazy backward redundant computation from the stashed FRC
 *            intermediates once the successor is preempted (Section 5.2 "Lazy
 *            BRC and Recovery"),
 *   failover merge of the victim's and the shadow's instruction groups
 *            (Section 5.2, rules 1-4).
 *
 * Conventions
 *   - Plain C types only.  "device" pointers are HIP device addresses owned by
 *     the caller; the library never allocates or frees device memory and keeps
 *     only the pointers.  "host" pointers are ordinary host memory.
 *   - Streams are hipStream_t values passed as void*; they stay the caller's.
 *   - Every compute call enqueues work and returns; nothing blocks the host
 *     except stage_sync (and stage_init, once per process, see there).  Calls on one stage must come from one host thread.
 *   - Return value: 0 (BAMBOO_OK) or a negative bamboo_status; no exception
 *     crosses this boundary and nothing aborts.
 *   - Tensors are row-major [tokens, features], tokens = micro_batch * seq,
 *     token t = sample (t / seq), position (t % seq).
 */
#ifndef BAMBOO_STAGE_H
#define BAMBOO_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bamboo_stage bamboo_stage_t; /* opaque, host side */

enum bamboo_status {
  BAMBOO_OK = 0,
  BAMBOO_E_BADCFG = -1, /* configuration rejected (e.g. heads does not divide hidden) */
  BAMBOO_E_BADMB = -2,  /* micro-batch id out of range, or no stashed forward for it */
  BAMBOO_E_STATE = -3,  /* call not valid in the stage's current state */
  BAMBOO_E_HIP = -4,    /* a HIP runtime call failed */
  BAMBOO_E_ARG = -5,    /* null pointer, too small a buffer, misaligned pointer */
  BAMBOO_E_NOMEM = -6   /* host allocation failed */
};

enum bamboo_arch {
  BAMBOO_ARCH_POST_LN_ENCODER = 0, /* r1 = x + attn(x); y1 = LN1(r1); r2 = y1 + ffn(y1); y = LN2(r2) */
  BAMBOO_ARCH_PRE_LN_CAUSAL = 1    /* u = LN1(x); x1 = x + attn(u); v = LN2(x1); y = x1 + ffn(v); causal mask */
};

enum bamboo_dtype {
  BAMBOO_F32 = 0, /* fp32 weights, activations, arithmetic */
  BAMBOO_BF16 = 1 /* bf16 weights and activations, fp32 accumulation, fp32 gradients */
};

/* Redundant-computation variants (Section 7.4, Table 4).  Bamboo's design is eager FRC + lazy
 * BRC; the other two are what the paper measures it against.
 *   LFLB  nothing redundant runs until a preemption; the failover schedule then runs FRC before
 *         every BRC (longer pause).  Also the setting for "redundancy off" (the schedule is the same).
 *   EFLB  FRC(k) on lane 1 right after FWD(k); BRC only after a preemption.
 *   EFEB  as EFLB, and BRC(k) on lane 1 as soon as the upstream gradient of the successor's layers
 *         exists (where the stage starts to wait for the successor's backward of micro-batch k);
 *         after a preemption nothing has to be replayed. */
enum bamboo_rc_mode { BAMBOO_RC_LFLB = 0, BAMBOO_RC_EFLB = 1, BAMBOO_RC_EFEB = 2 };

/* Configuration of one stage (Section 4: the schedule is a static function of
 * the stage id, the pipeline depth and the number of micro-batches). */
typedef struct {
  int32_t arch;        /* enum bamboo_arch */
  int32_t dtype;       /* enum bamboo_dtype */
  int32_t hidden;      /* H, multiple of 8 */
  int32_t heads;       /* divides H; head size H/heads <= 128 */
  int32_t ffn;         /* F, multiple of 8 */
  int32_t seq;         /* S */
  int32_t micro_batch; /* samples per micro-batch */
  int32_t n_own;       /* layers of this stage */
  int32_t n_shadow;    /* replica layers of the successor (0: no redundancy) */
  int32_t P;           /* pipeline depth */
  int32_t stage_id;    /* 0-indexed forward stage id (Section 5.1) */
  int32_t M;           /* micro-batches per iteration, <= 32767 */
  int32_t rc_mode;     /* enum bamboo_rc_mode: which redundant computation runs eagerly */
  int32_t tick_F;      /* slot-timeline duration of a forward (>= 1) */
  int32_t tick_B;      /* slot-timeline duration of a backward (>= 1) */
  float ln_eps;        /* LayerNorm epsilon */
  int32_t swap_slots;  /* 0: FRC results stay in device memory (M shadow stash slots).  R in 1..M: the
                          paper's swap-out (Section 5.2): the device keeps a ring of R shadow slots, the
                          results of every FRC are copied to pinned host memory on a third stream and copied
                          back only for BRC.  Needs stage_swap_attach before the first FRC. */
  int32_t wrap;        /* 1: this is the last stage (stage_id == P-1) and its replica layers are the FIRST
                          stage's (Section 5.1: the last node is the first node's predecessor and fetches
                          the input samples itself).  FRC(k) then does not depend on FWD(k), and the
                          failover schedule is the wrap-around one.  rc_mode EFLB or LFLB.  0 otherwise. */
  int32_t data_parallel; /* 1: pure data parallelism (Section 5.2, "Support for Pure Data Parallelism"): the
                          node holds the whole model (P == 1, stage_id == 0) and its replica layers are a
                          copy of ANOTHER node's model (n_shadow == n_own).  There is no bubble: eager FRC
                          is "over-batching", FRC(k) runs the other node's micro-batch k (the caller passes
                          it as `y`) beside the node's own and does not depend on FWD(k); BRC(k) takes
                          the other node's upstream gradient.  rc_mode LFLB or EFLB.  0 otherwise. */
} bamboo_cfg_t;

/* Instruction set: the paper's computation and communication instructions
 * (Section 4) plus FRC/BRC, the simulated bubble and the join of the two lanes. */
enum bamboo_op {
  BAMBOO_RECV_ACT = 0,
  BAMBOO_SEND_ACT = 1,
  BAMBOO_RECV_GRAD = 2,
  BAMBOO_SEND_GRAD = 3,
  BAMBOO_FWD = 4,
  BAMBOO_BWD = 5,
  BAMBOO_FRC = 6,
  BAMBOO_BRC = 7,
  BAMBOO_BUBBLE = 8,
  BAMBOO_JOIN = 9,
  BAMBOO_ALLREDUCE = 10,
  BAMBOO_APPLY = 11
};

/* lane: 0 main stream, 1 FRC stream.  mb: micro-batch or -1.
 * arg: FWD/BWD own stash slot (mb mod c_own); FRC/BRC shadow stash slot (mb);
 *      communication: peer stage id; BUBBLE: ticks; JOIN: last FRC waited for
 *      (-1 all); otherwise 0. */
typedef struct {
  uint8_t op;
  uint8_t lane;
  int16_t mb;
  int32_t arg;
} bamboo_instr_t;

/* Buffer sizes in bytes the caller must provide for a configuration. */
typedef struct {
  uint64_t own_w, shadow_w;         /* parameters in the storage dtype */
  uint64_t own_g, shadow_g;         /* fp32 gradients, same element layout */
  uint64_t own_stash, shadow_stash; /* c_own (c_shadow) slots x layers x rec_bytes */
  uint64_t workspace;               /* scratch for both lanes */
  uint64_t rec_bytes;               /* one stash record: one layer, one micro-batch */
  uint64_t layer_params;            /* elements per layer: 4H^2 + 2HF + 9H + F */
  int32_t c_own;                    /* own stash slots = min(P - stage_id, M) */
  int32_t c_shadow;                 /* shadow stash slots in device memory = M (everything BRC may need),
                                       or cfg.swap_slots when the FRC results are swapped out to the host */
  uint64_t own_opt, shadow_opt;     /* optimizer state (only for stage_optimizer_init): fp32 master weights,
                                       first and second moments, 3 x 4 bytes per parameter */
  uint64_t host_stash;              /* pinned host bytes for stage_swap_attach: M x n_shadow x rec_bytes
                                       (0 when cfg.swap_slots is 0) */
} bamboo_sizes_t;

/* Adam hyper-parameters (Section 7 names the optimizer and a learning rate of 6e-3 for the
 * language models; beta1 0.9, beta2 0.999, eps 1e-8 are the usual defaults). */
typedef struct {
  float lr, beta1, beta2, eps;
} bamboo_adam_t;

/* ---- host-only entry points (no GPU needed) ------------------------------ */

/* Validate cfg and report buffer sizes.  host pointers. */
int stage_query_sizes(const bamboo_cfg_t* cfg, bamboo_sizes_t* out);

/* The stage's instruction list for one failure-free iteration: 1F1B with flush
 * (Section 2), groups of leading communication + computation (Section 5.2),
 * BUBBLE(ticks) where the zero-latency slot timeline of all P stages leaves the
 * stage idle, FRC(k) on lane 1 right after FWD(k) and before the stage talks to
 * its successor (Section 5.2 "Scheduling").  out: host array of cap entries, may
 * be NULL with cap 0 to ask for the count.  Returns the count or a negative
 * status; BAMBOO_E_ARG if cap is too small. */
int stage_program(const bamboo_cfg_t* cfg, bamboo_instr_t* out, int32_t cap);

/* stage_program for a pipeline whose stages differ in speed (Section 5.2: the partition gives
 * later stages more layers, so they are slower and earlier stages see larger bubbles):
 * tick_F[P], tick_B[P] are the slot-timeline durations of a forward / backward on each stage
 * (host arrays; NULL = cfg->tick_F / cfg->tick_B for every stage).  Only the BUBBLE instructions
 * differ from stage_program's. */
int stage_program_uneven(const bamboo_cfg_t* cfg, const int32_t* tick_F, const int32_t* tick_B, bamboo_instr_t* out,
                         int32_t cap);

/* The failover schedule of the shadow stage when sending micro-batch k_fail's
 * activation to the successor fails (Section 5.2, merge rules 1-4): join the FRC
 * lane, replay BRC for the micro-batches whose successor-side gradients were
 * lost, then the rest of the 1F1B program with the victim's groups merged in.
 * Same out/cap/return convention as stage_program. */
int stage_failover_program(const bamboo_cfg_t* cfg, int32_t k_fail, bamboo_instr_t* out, int32_t cap);

/* A whole iteration of the stage AFTER it has taken over the victim's layers (Section 5.2: until the
 * pipeline is reconfigured, the shadow node executes all of the victim's instructions): the stage's
 * own 1F1B order with the victim's computation of the same micro-batch merged in under rules 1-4
 * -- the last part of stage_failover_program started at the first computation, with nothing to
 * join and nothing to replay; FRC and BRC run on lane 0; no bubbles are simulated.  With cfg.wrap:
 * both ends' computations merged by failure-free start time as in the wrap-around failover
 * schedule.  With cfg.data_parallel: both nodes' minibatches, no communication.  Same
 * out/cap/return convention as stage_program; BAMBOO_E_STATE where there is nothing to take over. */
int stage_merged_program(const bamboo_cfg_t* cfg, bamboo_instr_t* out, int32_t cap);

/* With cfg.wrap the victim is the first stage and the shadow the last.  The two are the two ends of
 * the pipeline, so no traffic between them turns internal (unless P == 2).  stage_failover_program
 * then returns: JOIN up to FRC(k_fail); BRC replay of the micro-batches the victim had
 * back-propagated (their gradients come again from the second stage); then everything either
 * stage still has to do, merged by start time on the failure-free slot timeline (ties: backward
 * before forward, the victim's before the shadow's own).  The victim's forwards are FRCs on the
 * fetched samples, all still to do beyond k_fail; their outputs are sent to the second stage
 * only where the victim had not delivered them.
 * stage_wrap_victim_progress: how many forwards / backwards the first stage had finished on that
 * timeline when the last stage finishes FWD(k_fail) (host int32 outputs). */
int stage_wrap_victim_progress(const bamboo_cfg_t* cfg, int32_t k_fail, int32_t* n_fwd, int32_t* n_bwd);

/* Byte offset of stash record (slot, layer) inside a stash arena:
 * (slot * n_layers + layer) * rec_bytes.  kind 0 own, 1 shadow.  Negative status
 * on a bad index. */
int64_t stage_record_offset(const bamboo_cfg_t* cfg, int32_t kind, int32_t slot, int32_t layer);

/* Byte offsets of the tensors inside one stash record (everything the backward
 * of one layer needs for one micro-batch), so that a caller can inspect the stash:
 * out[0] x      layer input [T,H]
 * out[1] ain    attention input [T,H] (pre-LN: LN1(x); post-LN: same offset as x)
 * out[2] qkv    [T,3H]      out[3] ctx [T,H] (attention output before Wo)
 * out[4] r1     x + attention block [T,H]
 * out[5] fin    FFN input [T,H] (post-LN: LN1(r1); pre-LN: LN2(r1))
 * out[6] g      GELU(h) [T,F], h = fin W1 + b1 the FFN pre-activation (not kept itself)
 * out[7] dg     GELU'(h) [T,F]: what the backward multiplies the gradient of g by
 * out[8] r2     post-LN only: fin + ffn [T,H] (0 otherwise)
 * out[9] lse    fp32 [batch,heads,seq]   out[10], out[11] LN1, LN2 (mean, rstd) fp32 [T,2]
 * out[12] rec_bytes.  Activations are in the storage dtype.  host pointers. */
int stage_record_fields(const bamboo_cfg_t* cfg, uint64_t out[13]);

const char* stage_strerror(int status);

/* ---- stage object --------------------------------------------------------- */

/* Create a stage.  All device buffers must be at least as large as
 * stage_query_sizes reports and 256-byte aligned.
 *   own_w, shadow_w   device, read-only: layers concatenated in forward order,
 *                     each layer = Wqkv[H,3H] bqkv[3H] Wo[H,H] bo[H] g1[H] be1[H]
 *                     W1[H,F] b1[F] W2[F,H] b2[H] g2[H] be2[H]; matrices are
 *                     [in,out] row-major (Y = X W); Wqkv columns [0,H) queries,
 *                     [H,2H) keys, [2H,3H) values, head h = columns h*d..(h+1)*d-1
 *                     of each third.  shadow_w holds the successor's values
 *                     (Section 5.1: same parameters); NULL iff n_shadow == 0.
 *   own_g, shadow_g   device fp32, same element layout; the library only adds
 *                     to them, the caller zeroes them at the start of an iteration.
 *   stashes, workspace device scratch owned by the caller for the stage's life.
 *   stream_main/frc   hipStream_t of lane 0 and lane 1 (default priority).
 * The replica is assumed equal to the successor's parameters at iteration start.
 * The first stage_init of a process with the bf16 dtype fills a 30 KB device table (GELU lookup)
 * on stream_main and waits for it: set-up is the one place that blocks, so that no compute call does. */
int stage_init(const bamboo_cfg_t* cfg, const bamboo_sizes_t* sizes, const void* own_w, const void* shadow_w,
               void* own_g, void* shadow_g, void* own_stash, void* shadow_stash, void* workspace,
               void* stream_main, void* stream_frc, bamboo_stage_t** out);

/* Copy the current instruction list (stage_program, or the failover schedule
 * once failover_merge has been called).  Same convention as stage_program. */
int stage_schedule(const bamboo_stage_t* st, bamboo_instr_t* out, int32_t cap);

/* Forget all stash contents and events: start of a new iteration.  Does not
 * touch gradients.  After failover_merge the stage stays merged, and from the first
 * stage_begin_iteration after the merge on stage_schedule returns stage_merged_program. */
int stage_begin_iteration(bamboo_stage_t* st);

/* FNC_s(k): y = own layers(x) on lane 0; intermediates go to own slot k mod c_own.
 * x, y device [tokens, H] in the storage dtype.  BAMBOO_E_BADMB if k is outside
 * [0, M) or its slot still holds a forward that has not been back-propagated. */
int stage_fwd(bamboo_stage_t* st, int32_t k, const void* x, void* y);

/* FRC(k): z = shadow layers(y) on lane 1 (lane 0 after failover_merge), ordered
 * after stage_fwd(k) by an event; intermediates go to shadow slot k and stay
 * until BRC(k) or the next iteration.  z (device, [tokens,H]) may be NULL.  y
 * must stay untouched until FRC(k) has run.  BAMBOO_E_STATE if n_shadow == 0 or
 * FRC is disabled; BAMBOO_E_BADMB if stage_fwd(k) was not issued or FRC(k)
 * already was. */
int shadow_fwd_frc(bamboo_stage_t* st, int32_t k, const void* y, void* z);

/* BNC_s(k): gx = own backward(gy) on lane 0 from own slot k mod c_own; own_g +=.
 * Frees the slot. */
int stage_bwd(bamboo_stage_t* st, int32_t k, const void* gy, void* gx);

/* BRC(k): gy = shadow backward(gz) from shadow slot k; shadow_g +=.  gy may be NULL (a replayed
 * micro-batch whose own backward already ran, or eager BRC beside a live successor, whose g_y is the
 * successor's to deliver).  Lazy BRC (rc_mode LFLB, EFLB; Section 5.2) is valid only after
 * failover_merge and runs on lane 0, behind the FRC of the same micro-batch.  Eager BRC (rc_mode
 * EFEB; Section 7.4) is also valid before a preemption and then runs on lane 1, behind FRC(k) in
 * that lane's order; after failover_merge it runs on lane 0 like the lazy one.  BAMBOO_E_STATE when
 * neither applies or slot k holds no FRC results.  Frees the slot. */
int shadow_bwd_brc(bamboo_stage_t* st, int32_t k, const void* gz, void* gy);

/* The successor was found dead while handing over micro-batch k_fail: lane 0
 * waits for the FRC lane, the stage switches to merged mode (FRC on lane 0, BRC
 * allowed) and the failover schedule is written to out (host array of cap entries).
 * BAMBOO_E_STATE when called twice or with n_shadow == 0; BAMBOO_E_ARG when out is
 * NULL or cap is too small -- the stage is then left as it was (ask
 * stage_failover_program for the count beforehand: it has no side effects).
 * Returns the instruction count. */
int failover_merge(bamboo_stage_t* st, int32_t k_fail, bamboo_instr_t* out, int32_t cap);

/* ---- interpreting an instruction list inside the library ---------------------------------
 * Section 4: a worker interprets its static schedule, instruction by instruction; a communication
 * instruction is where a lost neighbour shows.  stage_run does that for a list produced by
 * stage_schedule / failover_merge: every computation instruction becomes the call named beside it,
 * on the buffers of its micro-batch; communication instructions, which on one GPU move nothing,
 * are handed to the caller's hook, which stands for the neighbours.
 *   FWD(k)  stage_fwd(k, x[k], y[k])
 *   FRC(k)  shadow_fwd_frc(k, frc_in ? frc_in[k] : y[k], z ? z[k] : NULL)
 *   BWD(k)  stage_bwd(k, gy[k], gx[k])
 *   BRC(k)  before a merge (eager BRC beside a live successor): shadow_bwd_brc(k, gz[k], NULL);
 *           after it: shadow_bwd_brc(k, gz[k], gy[k]) -- the gradient the victim would have sent --
 *           unless BWD(k) already ran in this iteration (a replayed micro-batch) or the victim is a
 *           data-parallel peer (its input gradient feeds nothing here): then the output goes to
 *           gy_replay[k], or nowhere if gy_replay is NULL
 *   BUBBLE  stage_bubble(ticks, us_per_tick) if us_per_tick > 0       JOIN  stage_join
 *   APPLY   stage_apply(adam, ++step) if adam != NULL and stage_optimizer_init has been called
 *   RECV_ACT, SEND_ACT, RECV_GRAD, SEND_GRAD, ALLREDUCE: comm(user, &instruction) if comm != NULL;
 *           a nonzero return means the peer is gone: stage_run stops BEFORE that instruction and
 *           returns its index, and the caller goes on with failover_merge.
 * All table entries are device pointers to [tokens, hidden] tensors in the storage dtype, M per
 * table, owned by the caller; tables whose instructions do not occur in the list may be NULL
 * (BAMBOO_E_ARG if one that is needed is).  BAMBOO_E_STATE for a stage with cfg.wrap, whose
 * instructions are pairs of calls into the stage and the model's ends (bamboo_ends.h) that the
 * caller composes.  Returns n when the whole list has been issued, the
 * index of the refused communication instruction, or a negative status from the failing call. */
typedef int (*bamboo_comm_fn)(void* user, const bamboo_instr_t* instr);
typedef struct {
  const void* const* x;       /* inputs of FWD (stand for RECV_ACT from stage s-1) */
  void* const* y;             /* outputs of FWD */
  const void* const* frc_in;  /* inputs of FRC when they are not y (data parallel: the peer's minibatch), or NULL */
  void* const* z;             /* outputs of FRC, or NULL */
  void* const* gy;            /* gradients at y: read by BWD; written by BRC once merged */
  void* const* gx;            /* outputs of BWD */
  const void* const* gz;      /* upstream gradients of the replica's layers, read by BRC */
  void* const* gy_replay;     /* outputs of replayed BRCs, or NULL */
  float us_per_tick;          /* length of one simulated bubble tick; 0: bubbles are skipped */
  const bamboo_adam_t* adam;  /* hyper-parameters for APPLY, or NULL: APPLY is skipped */
  bamboo_comm_fn comm;        /* hook for communication instructions, or NULL */
  void* user;
} bamboo_tables_t;
int stage_run(bamboo_stage_t* st, const bamboo_instr_t* program, int32_t n, const bamboo_tables_t* tables);

/* ---- the APPLY instruction and the replica's weight synchronisation ----------------------
 * Section 5.1: node n keeps a replica of node n+1's layers together with their optimizer state,
 * and FRC/BRC use the same parameters as node n+1.  The paper gives no mechanism; here the
 * replica is overwritten with the successor's values after every update.
 *
 * stage_optimizer_init: own_opt / shadow_opt are device buffers of sizes.own_opt / sizes.shadow_opt
 * bytes (256-byte aligned; shadow_opt may be NULL when n_shadow == 0), laid out as
 * [master | m | v], each layer_params * n_layers floats in parameter order.  Enqueues on lane 0:
 * master <- the current parameters widened to fp32, m = v = 0.  From then on own_w (and shadow_w)
 * passed to stage_init are rewritten by stage_apply / stage_sync_replica although stage_init took
 * them as const. */
int stage_optimizer_init(bamboo_stage_t* st, void* own_opt, void* shadow_opt);

/* APPLY: one Adam step (step counts from 1) on the own parameters from the own gradients, on
 * lane 0.  After failover_merge the stage owns the victim's layers too: the replica parameters
 * are then updated from the replica gradients with the replica's optimizer state.
 * BAMBOO_E_STATE without stage_optimizer_init. */
int stage_apply(bamboo_stage_t* st, const bamboo_adam_t* hp, int32_t step);

/* Replica weight synchronisation, on lane 0: the replica parameters become successor_w (device,
 * sizes.shadow_w bytes: the successor's own parameters after its update) and, if successor_opt is
 * not NULL, the replica's optimizer state becomes successor_opt (device, sizes.shadow_opt bytes).
 * Stands for the transfer from node n+1 to node n; on one GPU it is a device-local copy. */
int stage_sync_replica(bamboo_stage_t* st, const void* successor_w, const void* successor_opt);

/* ---- swap-out of the FRC results to host memory (Section 5.2, "Eager FRC") ------------------
 * The paper moves the outputs and intermediate results of each micro-batch's FRC to CPU memory
 * right after the FRC and keeps only the replica's parameters on the GPU; they come back only
 * when a preemption makes BRC necessary.  With cfg.swap_slots = R > 0 the shadow stash passed to
 * stage_init holds R micro-batch slots (FRC(k) writes slot k mod R) and
 *   - after FRC(k), the swap stream waits for it and copies the slot to host_stash[k]; a later FRC
 *     into the same slot waits for that copy;
 *   - BRC(k) reads the slot directly if it still holds k, else the swap stream copies host_stash[k]
 *     back first; while BRC(k) runs, the copy for the next BRC of the stage's program is started
 *     when it lands in another slot.
 * host_stash: page-locked host memory of sizes.host_stash bytes (micro-batch k at offset
 * k * n_shadow * rec_bytes, records in layer order), allocated pinned by the caller (not
 * registered after the fact) and kept until stage_destroy.  stream_swap: a third stream of the
 * same priority as the other two.  BAMBOO_E_STATE if cfg.swap_slots == 0 or already attached;
 * BAMBOO_E_ARG if bytes is too small.  Results are bitwise those of the device-resident stash. */
int stage_swap_attach(bamboo_stage_t* st, void* host_stash, uint64_t bytes, void* stream_swap);

/* Simulated pipeline bubble: one single-wave workgroup on lane 0 that spins on
 * the device wall clock for ticks * us_per_tick microseconds. */
int stage_bubble(bamboo_stage_t* st, int32_t ticks, float us_per_tick);

/* JOIN on the device: lane 0 waits for everything issued on lane 1 (and on the swap stream). */
int stage_join(bamboo_stage_t* st);

/* JOIN and block the host until all lanes are idle. */
int stage_sync(bamboo_stage_t* st);

int stage_destroy(bamboo_stage_t* st);

#ifdef __cplusplus
}
#endif
#endif /* BAMBOO_STAGE_H */
