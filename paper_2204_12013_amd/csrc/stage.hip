// Stage object and the C ABI: host orchestration of the Bamboo stage hot path.
//
// Lane 0 (main stream) carries FNC/BNC of the stage's own layers and, after a
// failover, BRC and FRC as well.  Lane 1 (FRC stream) carries the eager forward
// redundant computation over the successor's replica layers, ordered after the
// forward of the same micro-batch by an event, so that it falls into whatever
// the main lane leaves idle (a bubble) or overlaps the next forward (paper
// Section 5.2).  FRC intermediates stay in an HBM stash (one slot per
// micro-batch) until BRC consumes them; the paper swaps them to host memory
// instead, which 288 GB of HBM makes unnecessary.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "../../include/bamboo_debug.h"
#include "common.h"
#include "schedule.h"

using namespace bamboo;

namespace {

constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Byte offsets of the named tensors inside one layer's parameter vector.
struct ParamOffsets {
  uint64_t Wqkv, bqkv, Wo, bo, g1, be1, W1, b1, W2, b2, g2, be2, count;
};
ParamOffsets param_offsets(int H, int F) {
  ParamOffsets p;
  uint64_t o = 0;
  p.Wqkv = o; o += (uint64_t)H * 3 * H;
  p.bqkv = o; o += 3 * (uint64_t)H;
  p.Wo = o; o += (uint64_t)H * H;
  p.bo = o; o += H;
  p.g1 = o; o += H;
  p.be1 = o; o += H;
  p.W1 = o; o += (uint64_t)H * F;
  p.b1 = o; o += F;
  p.W2 = o; o += (uint64_t)F * H;
  p.b2 = o; o += H;
  p.g2 = o; o += H;
  p.be2 = o; o += H;
  p.count = o;
  return p;
}

// One stash record = everything the backward of one layer needs for one
// micro-batch.  Probabilities are not kept (recomputed from the log-sum-exp).
//   x     layer input                      [T,H]
//   ain   attention input (pre-LN: LN1(x); post-LN: aliases x)
//   qkv   projected queries|keys|values    [T,3H]
//   ctx   attention output before Wo       [T,H]
//   r1    x + attention block              [T,H]   (post-LN: LN1 input, pre-LN: x1)
//   fin   FFN input (post-LN: y1 = LN1(r1); pre-LN: v = LN2(x1))
//   g     GELU(h), h = fin W1 + b1         [T,F]   (the FFN pre-activation h itself is not kept:
//   dg    GELU'(h)                         [T,F]    the forward evaluates GELU and its derivative once)
//   r2    post-LN only: y1 + ffn, LN2 input [T,H]
//   lse, ln1, ln2  fp32 side data
struct RecordLayout {
  uint64_t x, ain, qkv, ctx, r1, fin, g, dg, r2, lse, ln1, ln2, bytes;
};
RecordLayout record_layout(const bamboo_cfg_t& c) {
  const uint64_t es = c.dtype == BAMBOO_BF16 ? 2 : 4;
  const uint64_t T = (uint64_t)c.micro_batch * c.seq, H = c.hidden, F = c.ffn;
  RecordLayout r;
  uint64_t o = 0;
  r.x = o; o = align_up(o + T * H * es);
  if (c.arch == BAMBOO_ARCH_PRE_LN_CAUSAL) { r.ain = o; o = align_up(o + T * H * es); } else { r.ain = r.x; }
  r.qkv = o; o = align_up(o + T * 3 * H * es);
  r.ctx = o; o = align_up(o + T * H * es);
  r.r1 = o; o = align_up(o + T * H * es);
  r.fin = o; o = align_up(o + T * H * es);
  r.g = o; o = align_up(o + T * F * es);
  r.dg = o; o = align_up(o + T * F * es);
  if (c.arch == BAMBOO_ARCH_POST_LN_ENCODER) { r.r2 = o; o = align_up(o + T * H * es); } else { r.r2 = 0; }
  r.lse = o; o = align_up(o + (uint64_t)c.micro_batch * c.heads * c.seq * 4);
  r.ln1 = o; o = align_up(o + 2 * T * 4);
  r.ln2 = o; o = align_up(o + 2 * T * 4);
  r.bytes = o;
  return r;
}

// Scratch of one lane.  Lane 1 only ever runs forwards: it needs only out (where an
// output the caller does not want is written).
struct LaneScratch {
  uint64_t out, dh, d1, d2, d3, dctx, ping, pong, dqkv, delta, bytes;
  // partial rows of one layer's parameter-gradient reductions (summed by one launch at the layer's end):
  // LayerNorm 1 and 2 (gain, shift, column sums of the output), and the column sums of dh, dqkv, df
  uint64_t p_ln[2][3], p_dh, p_dqkv, p_df;
};
LaneScratch lane_scratch(const bamboo_cfg_t& c, bool backward) {
  const uint64_t es = c.dtype == BAMBOO_BF16 ? 2 : 4;
  const uint64_t T = (uint64_t)c.micro_batch * c.seq, H = c.hidden, F = c.ffn;
  LaneScratch w;
  memset(&w, 0, sizeof(w));
  uint64_t o = 0;
  w.out = o; o = align_up(o + T * H * es);
  if (backward) {
    w.dh = o; o = align_up(o + T * F * es);
    w.d1 = o; o = align_up(o + T * H * es);
    w.d2 = o; o = align_up(o + T * H * es);
    w.d3 = o; o = align_up(o + T * H * es);
    w.dctx = o; o = align_up(o + T * H * es);
    w.ping = o; o = align_up(o + T * H * es);
    w.pong = o; o = align_up(o + T * H * es);
    w.dqkv = o; o = align_up(o + T * 3 * H * es);
    w.delta = o; o = align_up(o + (uint64_t)c.micro_batch * c.heads * c.seq * 4);
    const uint64_t rows = reduce_max_partials();
    for (int a = 0; a < 2; ++a)
      for (int b = 0; b < 3; ++b) { w.p_ln[a][b] = o; o = align_up(o + rows * H * 4); }
    w.p_dh = o; o = align_up(o + rows * F * 4);
    w.p_dqkv = o; o = align_up(o + rows * 3 * H * 4);
    w.p_df = o; o = align_up(o + rows * H * 4);
  }
  w.bytes = o;
  return w;
}

int validate(const bamboo_cfg_t* c) {
  if (!c) return BAMBOO_E_ARG;
  if (c->arch != BAMBOO_ARCH_POST_LN_ENCODER && c->arch != BAMBOO_ARCH_PRE_LN_CAUSAL) return BAMBOO_E_BADCFG;
  if (c->dtype != BAMBOO_F32 && c->dtype != BAMBOO_BF16) return BAMBOO_E_BADCFG;
  if (c->hidden <= 0 || c->hidden % 8 || c->ffn <= 0 || c->ffn % 8) return BAMBOO_E_BADCFG;
  if (c->heads <= 0 || c->hidden % c->heads || c->hidden / c->heads > 128) return BAMBOO_E_BADCFG;
  if (c->seq <= 0 || c->micro_batch <= 0 || c->n_own <= 0 || c->n_shadow < 0) return BAMBOO_E_BADCFG;
  if (c->P <= 0 || c->stage_id < 0 || c->stage_id >= c->P || c->M <= 0 || c->M > 32767) return BAMBOO_E_BADCFG;
  if (c->tick_F < 1 || c->tick_B < 1 || !(c->ln_eps >= 0.f)) return BAMBOO_E_BADCFG;
  if (c->rc_mode != BAMBOO_RC_LFLB && c->rc_mode != BAMBOO_RC_EFLB && c->rc_mode != BAMBOO_RC_EFEB) return BAMBOO_E_BADCFG;
  if ((uint64_t)c->seq * c->micro_batch > (1u << 24)) return BAMBOO_E_BADCFG;
  if (c->swap_slots < 0 || c->swap_slots > c->M || (c->swap_slots > 0 && c->n_shadow <= 0)) return BAMBOO_E_BADCFG;
  if (c->wrap != 0 && c->wrap != 1) return BAMBOO_E_BADCFG;
  // The wrap-around stage runs the paper's own variant (eager FRC, lazy BRC) and the lazy one.  Eager BRC is
  // not offered there: the gradient it needs leaves the second stage a whole pipeline traversal after the
  // last stage's own backward, so "as soon as the upstream gradient exists" has no anchor in the last
  // stage's own instruction order -- it would have to be placed by simulated time, a scheduling policy
  // the paper (which measures the variants on middle stages, Section 7.4) does not describe.
  if (c->wrap && (c->P < 2 || c->stage_id != c->P - 1 || c->n_shadow <= 0 || c->rc_mode == BAMBOO_RC_EFEB))
    return BAMBOO_E_BADCFG;
  if (c->data_parallel != 0 && c->data_parallel != 1) return BAMBOO_E_BADCFG;
  // pure data parallelism: the whole model on one node, the replica is another node's model; the paper
  // describes eager FRC (over-batching) and lazy BRC for it, nothing eager on the backward side
  if (c->data_parallel && (c->P != 1 || c->wrap || c->n_shadow != c->n_own || c->rc_mode == BAMBOO_RC_EFEB))
    return BAMBOO_E_BADCFG;
  return BAMBOO_OK;
}

// whether the stage has a victim to take over: a successor, the first stage (wrap), a data-parallel peer
bool can_fail_over(const bamboo_cfg_t& c) {
  return c.n_shadow > 0 && (c.stage_id < c.P - 1 || c.wrap || c.data_parallel);
}
std::vector<bamboo_instr_t> failover_list(const bamboo_cfg_t& c, int k_fail) {
  return c.wrap ? build_wrap_failover_program(c, k_fail) : build_failover_program(c, k_fail);
}
std::vector<bamboo_instr_t> merged_list(const bamboo_cfg_t& c) {
  return c.wrap ? build_wrap_merged_program(c) : build_merged_program(c);
}

int copy_out(const std::vector<bamboo_instr_t>& v, bamboo_instr_t* out, int32_t cap) {
  if (out == nullptr && cap == 0) return (int)v.size();
  if (out == nullptr || cap < (int32_t)v.size()) return BAMBOO_E_ARG;
  memcpy(out, v.data(), v.size() * sizeof(bamboo_instr_t));
  return (int)v.size();
}

}  // namespace

struct bamboo_stage {
  bamboo_cfg_t cfg;
  bamboo_sizes_t sizes;
  ParamOffsets po;
  RecordLayout rl;
  LaneScratch ws0, ws1;
  const char* w[2];   // own, shadow parameters
  float* g[2];        // own, shadow gradients
  char* stash[2];
  char* wsbase;
  hipStream_t lane[2];
  std::vector<bamboo_instr_t> program;
  bool merged;
  std::vector<int> own_slot_mb;        // micro-batch stashed in each own slot, -1 free
  std::vector<char> fwd_issued, frc_issued, shadow_live, bwd_done;
  bool merged_program_installed;       // program is the merged stage's whole iteration (not a failover list)
  int apply_step;                      // optimizer steps taken through stage_run
  std::vector<hipEvent_t> ev_fwd, ev_frc;
  hipEvent_t ev_join;
  int last_frc_on_lane1;
  float* opt[2];      // own, shadow optimizer state [master | m | v], or null
  // swap-out of the FRC results (cfg.swap_slots = R > 0): the shadow stash is a ring of R slots
  char* host_stash;                    // pinned host memory, micro-batch k at k * n_shadow * rec_bytes; null until attached
  hipStream_t lane_swap;
  std::vector<int> ring_mb;            // micro-batch whose record the enqueued work leaves in each ring slot, -1 none
  std::vector<char> on_host;           // swap-out of micro-batch k has been enqueued
  std::vector<hipEvent_t> ev_written;  // per ring slot: last FRC into it
  std::vector<hipEvent_t> ev_out;      // per ring slot: last copy to the host out of it
  std::vector<hipEvent_t> ev_in;       // per ring slot: last copy from the host into it
  std::vector<hipEvent_t> ev_read;     // per ring slot: last BRC reading it
  hipEvent_t ev_swap_join;
  // optional per-kernel-class timing: an event pair around every launch
  bool prof_on;
  struct ProfRec { int cls; double work; hipEvent_t a, b; };
  std::vector<ProfRec> prof_recs;
  std::vector<hipEvent_t> prof_pool;
};

namespace {

#define HIPCHK(expr)                                                                          \
  do {                                                                                        \
    const hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) {                                                                   \
      if (getenv("BAMBOO_DEBUG"))                                                             \
        fprintf(stderr, "[bamboo] %s:%d HIP error %d: %s\n", __FILE__, __LINE__, (int)e_, hipGetErrorString(e_)); \
      (void)hipGetLastError();                                                                \
      return BAMBOO_E_HIP;                                                                    \
    }                                                                                         \
  } while (0)

// Brackets one launch (or a short fixed group of launches of one class) with an
// event pair on its stream when profiling is on.
struct ProfScope {
  bamboo_stage* st;
  hipStream_t s;
  hipEvent_t b;
  ProfScope(bamboo_stage* st_, int cls, hipStream_t s_, double work) : st(st_), s(s_), b(nullptr) {
    if (!st->prof_on) return;
    hipEvent_t ev[2] = {nullptr, nullptr};
    for (int i = 0; i < 2; ++i) {
      if (!st->prof_pool.empty()) {
        ev[i] = st->prof_pool.back();
        st->prof_pool.pop_back();
      } else if (hipEventCreate(&ev[i]) != hipSuccess) {
        (void)hipGetLastError();
        return;
      }
    }
    if (hipEventRecord(ev[0], s) != hipSuccess) (void)hipGetLastError();
    st->prof_recs.push_back({cls, work, ev[0], ev[1]});
    b = ev[1];
  }
  ~ProfScope() {
    if (b && hipEventRecord(b, s) != hipSuccess) (void)hipGetLastError();
  }
};

double gemm_flops(const GemmDesc& d) { return 2.0 * d.M * d.N * d.K; }

uint64_t esize(const bamboo_stage* st) { return st->cfg.dtype == BAMBOO_BF16 ? 2 : 4; }


#define BBCHK(expr)                 \
  do {                              \
    const int rc_ = (expr);         \
    if (rc_ != BAMBOO_OK) return rc_; \
  } while (0)

enum KernelClass {
  K_GEMM_QKV = BAMBOO_K_GEMM_QKV, K_GEMM_ATTN_OUT = BAMBOO_K_GEMM_ATTN_OUT, K_GEMM_FFN1 = BAMBOO_K_GEMM_FFN1,
  K_GEMM_FFN2 = BAMBOO_K_GEMM_FFN2, K_DGRAD_FFN2 = BAMBOO_K_DGRAD_FFN2, K_DGRAD_FFN1 = BAMBOO_K_DGRAD_FFN1,
  K_DGRAD_ATTN_OUT = BAMBOO_K_DGRAD_ATTN_OUT, K_DGRAD_QKV = BAMBOO_K_DGRAD_QKV, K_WGRAD_GROUP = BAMBOO_K_WGRAD_GROUP,
  K_ATTN_FWD = BAMBOO_K_ATTN_FWD, K_ATTN_BWD = BAMBOO_K_ATTN_BWD, K_LN_FWD = BAMBOO_K_LN_FWD,
  K_LN_BWD = BAMBOO_K_LN_BWD, K_COLSUM = BAMBOO_K_COLSUM, K_COUNT = BAMBOO_K_COUNT
};

// site: which GEMM of the layer pass this is (for the per-site timing)
int p_gemm(bamboo_stage* st, hipStream_t s, int site, const GemmDesc& d0) {
  GemmDesc d = d0;
  // Lane 1 runs beside lane 0, which is rarely idle: what its launches leave unused, lane 0 takes, so its forward
  // GEMMs are shaped for the least CU time.  Every tile shape gives the same output bits, so FRC still equals the
  // successor's forward; the input-gradient launches keep the one choice, because the column sums that ride in
  // their epilogue are partitioned by the tile rows.
  d.shared_chip = s == st->lane[1] && s != st->lane[0] && site <= K_GEMM_FFN2 ? 1 : 0;
  ProfScope ps(st, site, s, gemm_flops(d));
  HIPCHK(launch_gemm(s, st->cfg.dtype, d));
  return BAMBOO_OK;
}
// the weight-gradient GEMMs of one layer, as one launch where possible
// tail: reductions that may ride in the same launch; *tail_done tells whether they did
int p_gemm_group(bamboo_stage* st, hipStream_t s, const GemmDesc* d, int n, const GradReduceBatch* tail,
                 bool* tail_done) {
  double flops = 0;
  for (int i = 0; i < n; ++i) flops += gemm_flops(d[i]);
  ProfScope p(st, K_WGRAD_GROUP, s, flops);
  HIPCHK(launch_gemm_group(s, st->cfg.dtype, d, n, tail, tail_done));
  return BAMBOO_OK;
}
double attn_fwd_flops(const AttnDesc& a) {
  return 4.0 * a.B * a.heads * (double)a.S * a.S * a.d * (a.causal ? 0.5 : 1.0);
}
int p_attn_fwd(bamboo_stage* st, hipStream_t s, const AttnDesc& a) {
  ProfScope ps(st, K_ATTN_FWD, s, attn_fwd_flops(a));
  HIPCHK(launch_attention_fwd(s, st->cfg.dtype, a));
  return BAMBOO_OK;
}
int p_attn_bwd(bamboo_stage* st, hipStream_t s, const AttnDesc& a) {
  ProfScope ps(st, K_ATTN_BWD, s, 2.5 * attn_fwd_flops(a));
  HIPCHK(launch_attention_bwd(s, st->cfg.dtype, a));
  return BAMBOO_OK;
}
int p_ln_fwd(bamboo_stage* st, hipStream_t s, int T, int H, const void* r, const void* g, const void* b, void* y,
             float* stats) {
  ProfScope ps(st, K_LN_FWD, s, (double)T * (2.0 * H * esize(st) + 8.0));
  HIPCHK(launch_layernorm_fwd(s, st->cfg.dtype, T, H, st->cfg.ln_eps, r, g, b, y, stats));
  return BAMBOO_OK;
}
// LayerNorm backward: dr, plus partial rows of the gain / shift gradients and (pc != nullptr) of the
// column sums of dr; their ordered final sums into dgamma / dbeta / dbias are queued in `batch`
int p_ln_bwd(bamboo_stage* st, hipStream_t s, char* ws, int T, int H, const void* dout, const void* r, const float* stats,
             const void* gamma, const void* add, void* dr, float* dgamma, float* dbeta, float* dbias,
             const uint64_t (&poff)[3], GradReduceBatch* batch) {
  ProfScope ps(st, K_LN_BWD, s, (double)T * ((add ? 4.0 : 3.0) * H * esize(st) + 8.0));
  float* pg = (float*)(ws + poff[0]);      // ws: the scratch area of the lane the backward runs on
  float* pb = (float*)(ws + poff[1]);
  float* pc = dbias ? (float*)(ws + poff[2]) : nullptr;
  int parts = 0;
  HIPCHK(launch_layernorm_bwd_partials(s, st->cfg.dtype, T, H, dout, r, stats, gamma, add, dr, pg, pb, pc, &parts));
  if (!grad_reduce_add(batch, H, parts, pg, dgamma, pb, dbeta)) return BAMBOO_E_STATE;
  if (dbias && !grad_reduce_add(batch, H, parts, pc, dbias, nullptr, nullptr)) return BAMBOO_E_STATE;
  return BAMBOO_OK;
}
// partial rows of the column sums of a[T,N]; the final sum into `out` is queued in `batch`
int p_colsum(bamboo_stage* st, hipStream_t s, char* ws, int T, int N, const void* a, float* out, uint64_t poff,
             GradReduceBatch* batch) {
  ProfScope ps(st, K_COLSUM, s, (double)T * N * esize(st));
  float* p = (float*)(ws + poff);
  int parts = 0;
  HIPCHK(launch_colsum_partials(s, st->cfg.dtype, T, N, a, p, &parts));
  if (!grad_reduce_add(batch, N, parts, p, out, nullptr, nullptr)) return BAMBOO_E_STATE;
  return BAMBOO_OK;
}
int p_grad_reduce(bamboo_stage* st, hipStream_t s, const GradReduceBatch& batch) {
  double bytes = 0.0;
  for (int i = 0; i < batch.n; ++i) bytes += (double)batch.seg[i].parts * batch.seg[i].N * 4.0 * (batch.seg[i].p1 ? 2 : 1);
  ProfScope ps(st, K_COLSUM, s, bytes);
  HIPCHK(launch_grad_reduce(s, batch));
  return BAMBOO_OK;
}

GemmDesc gemm_nn(const void* X, const void* W, void* Y, int T, int N, int K, int epi) {
  GemmDesc d;
  memset(&d, 0, sizeof(d));
  d.A = X; d.B = W; d.C = Y; d.M = T; d.N = N; d.K = K;
  d.a_sm = K; d.a_sk = 1; d.b_sk = N; d.b_sn = 1; d.epi = epi;
  return d;
}
// dX[T,Kw] = dY[T,Nw] * W[Kw,Nw]^T
GemmDesc gemm_nt(const void* dY, const void* W, void* dX, int T, int Kw, int Nw, int epi) {
  GemmDesc d;
  memset(&d, 0, sizeof(d));
  d.A = dY; d.B = W; d.C = dX; d.M = T; d.N = Kw; d.K = Nw;
  d.a_sm = Nw; d.a_sk = 1; d.b_sk = 1; d.b_sn = Nw; d.epi = epi;
  return d;
}
// dW[Kw,Nw] += X[T,Kw]^T * dY[T,Nw]
GemmDesc gemm_tn(const void* X, const void* dY, float* dW, int T, int Kw, int Nw) {
  GemmDesc d;
  memset(&d, 0, sizeof(d));
  d.A = X; d.B = dY; d.C = dW; d.M = Kw; d.N = Nw; d.K = T;
  d.a_sm = 1; d.a_sk = Kw; d.b_sk = Nw; d.b_sn = 1; d.epi = EPI_ACC_F32;
  return d;
}

// forward of one layer stack; kind 0 own, 1 shadow
int run_forward(bamboo_stage* st, int kind, int lane_id, int slot, const void* x, void* y) {
  const bamboo_cfg_t& c = st->cfg;
  const int n = kind == 0 ? c.n_own : c.n_shadow;
  const int T = c.micro_batch * c.seq, H = c.hidden, F = c.ffn;
  const uint64_t es = esize(st);
  hipStream_t s = st->lane[lane_id];
  (void)hipGetLastError();  // do not inherit an unrelated earlier error of this thread
  const RecordLayout& r = st->rl;
  char* rec0 = st->stash[kind] + (uint64_t)slot * n * r.bytes;
  HIPCHK(hipMemcpyAsync(rec0 + r.x, x, (uint64_t)T * H * es, hipMemcpyDeviceToDevice, s));
  for (int l = 0; l < n; ++l) {
    char* rec = rec0 + (uint64_t)l * r.bytes;
    const char* W = st->w[kind] + (uint64_t)l * st->po.count * es;
    auto P = [&](uint64_t off) { return (const void*)(W + off * es); };
    void* out = (l == n - 1) ? y : (void*)(rec + r.bytes + r.x);
    AttnDesc a;
    memset(&a, 0, sizeof(a));
    a.B = c.micro_batch; a.S = c.seq; a.heads = c.heads; a.d = H / c.heads;
    a.causal = c.arch == BAMBOO_ARCH_PRE_LN_CAUSAL;
    a.qkv = rec + r.qkv; a.ctx = rec + r.ctx; a.lse = (float*)(rec + r.lse);
    GemmDesc d;
    if (c.arch == BAMBOO_ARCH_PRE_LN_CAUSAL)
      BBCHK(p_ln_fwd(st, s, T, H, rec + r.x, P(st->po.g1), P(st->po.be1), rec + r.ain,
                                  (float*)(rec + r.ln1)));
    d = gemm_nn(rec + r.ain, P(st->po.Wqkv), rec + r.qkv, T, 3 * H, H, EPI_BIAS);
    d.bias = P(st->po.bqkv);
    BBCHK(p_gemm(st, s, K_GEMM_QKV, d));
    BBCHK(p_attn_fwd(st, s, a));
    d = gemm_nn(rec + r.ctx, P(st->po.Wo), rec + r.r1, T, H, H, EPI_BIAS_RES);
    d.bias = P(st->po.bo);
    d.res = rec + r.x;
    BBCHK(p_gemm(st, s, K_GEMM_ATTN_OUT, d));
    if (c.arch == BAMBOO_ARCH_POST_LN_ENCODER)
      BBCHK(p_ln_fwd(st, s, T, H, rec + r.r1, P(st->po.g1), P(st->po.be1), rec + r.fin,
                                  (float*)(rec + r.ln1)));
    else
      BBCHK(p_ln_fwd(st, s, T, H, rec + r.r1, P(st->po.g2), P(st->po.be2), rec + r.fin,
                                  (float*)(rec + r.ln2)));
    d = gemm_nn(rec + r.fin, P(st->po.W1), rec + r.dg, T, F, H, EPI_BIAS_GELU);
    d.bias = P(st->po.b1);
    d.aux_out = rec + r.g;
    BBCHK(p_gemm(st, s, K_GEMM_FFN1, d));
    if (c.arch == BAMBOO_ARCH_POST_LN_ENCODER) {
      d = gemm_nn(rec + r.g, P(st->po.W2), rec + r.r2, T, H, F, EPI_BIAS_RES);
      d.bias = P(st->po.b2);
      d.res = rec + r.fin;
      BBCHK(p_gemm(st, s, K_GEMM_FFN2, d));
      BBCHK(p_ln_fwd(st, s, T, H, rec + r.r2, P(st->po.g2), P(st->po.be2), out,
                                  (float*)(rec + r.ln2)));
    } else {
      d = gemm_nn(rec + r.g, P(st->po.W2), out, T, H, F, EPI_BIAS_RES);
      d.bias = P(st->po.b2);
      d.res = rec + r.r1;
      BBCHK(p_gemm(st, s, K_GEMM_FFN2, d));
    }
  }
  return BAMBOO_OK;
}

// backward of one layer stack; gx may be null (input gradient discarded).  Lane 1 only with eager BRC.
int run_backward(bamboo_stage* st, int kind, int lane_id, int slot, const void* gy, void* gx) {
  const bamboo_cfg_t& c = st->cfg;
  const int n = kind == 0 ? c.n_own : c.n_shadow;
  const int T = c.micro_batch * c.seq, H = c.hidden, F = c.ffn;
  const uint64_t es = esize(st);
  hipStream_t s = st->lane[lane_id];
  (void)hipGetLastError();
  char* ws = st->wsbase + (lane_id == 0 ? 0 : st->ws0.bytes);
  const LaneScratch& w = lane_id == 0 ? st->ws0 : st->ws1;
  void* dh = ws + w.dh;
  void* d1 = ws + w.d1;
  void* d2 = ws + w.d2;
  void* d3 = ws + w.d3;
  void* dctx = ws + w.dctx;
  void* dqkv = ws + w.dqkv;
  const RecordLayout& r = st->rl;
  char* rec0 = st->stash[kind] + (uint64_t)slot * n * r.bytes;
  const void* dy = gy;
  for (int l = n - 1; l >= 0; --l) {
    char* rec = rec0 + (uint64_t)l * r.bytes;
    const char* W = st->w[kind] + (uint64_t)l * st->po.count * es;
    float* G = st->g[kind] + (uint64_t)l * st->po.count;
    auto P = [&](uint64_t off) { return (const void*)(W + off * es); };
    void* dx = (l == 0) ? (gx ? gx : (void*)(ws + w.ping)) : (void*)(ws + (((n - 1 - l) & 1) ? w.pong : w.ping));
    if (dx == dy) dx = ws + w.pong;  // never alias input and output of a layer
    AttnDesc a;
    memset(&a, 0, sizeof(a));
    a.B = c.micro_batch; a.S = c.seq; a.heads = c.heads; a.d = H / c.heads;
    a.causal = c.arch == BAMBOO_ARCH_PRE_LN_CAUSAL;
    a.qkv = rec + r.qkv; a.ctx = rec + r.ctx; a.lse = (float*)(rec + r.lse);
    a.dctx = dctx; a.dqkv = dqkv; a.delta = (float*)(ws + w.delta);
    // Every reduction over tokens of this layer (LayerNorm gain / shift gradients, the four bias
    // gradients) leaves partial rows in the workspace; one launch at the end adds their ordered sums
    // to the gradients.  A bias gradient whose dY comes out of a LayerNorm backward is reduced there.
    GradReduceBatch batch;
    batch.n = 0;
    GemmDesc d;
    const void* df;     // gradient at the FFN output
    if (c.arch == BAMBOO_ARCH_POST_LN_ENCODER) {
      BBCHK(p_ln_bwd(st, s, ws, T, H, dy, rec + r.r2, (const float*)(rec + r.ln2), P(st->po.g2), nullptr, d3,
                     G + st->po.g2, G + st->po.be2, G + st->po.b2, w.p_ln[1], &batch));
      df = d3;
    } else {
      df = dy;
      BBCHK(p_colsum(st, s, ws, T, H, df, G + st->po.b2, w.p_df, &batch));
    }
    // f = g W2 + b2
    d = gemm_nt(df, P(st->po.W2), dh, T, F, H, EPI_MUL);   // through the activation: times GELU'(h)
    d.aux_in = rec + r.dg;
    // the column sums of dh (the gradient of b1) come out of the same kernel, one partial row per tile row
    // (as long as the smallest tile's rows, T / 64, fit the partial buffer)
    const bool fused_sum = (size_t)((T + 63) / 64) <= reduce_max_partials();
    int dh_parts = 0;
    if (fused_sum) {
      d.tile_colsum = (float*)(ws + w.p_dh);
      d.tile_colsum_parts = &dh_parts;
    }
    BBCHK(p_gemm(st, s, K_DGRAD_FFN2, d));
    if (fused_sum) {
      if (!grad_reduce_add(&batch, F, dh_parts, (const float*)(ws + w.p_dh), G + st->po.b1, nullptr, nullptr))
        return BAMBOO_E_STATE;
    } else {
      BBCHK(p_colsum(st, s, ws, T, F, dh, G + st->po.b1, w.p_dh, &batch));
    }
    // The four weight gradients of the layer wait until its end: their operands (df, dh, da, dqkv and the
    // record) all live that long, nothing in the layer depends on them, and launched together their tiles
    // share the rounds of the chip.
    GemmDesc wgrad[4];
    wgrad[0] = gemm_tn(rec + r.g, df, G + st->po.W2, T, F, H);
    // h = fin W1 + b1
    wgrad[1] = gemm_tn(rec + r.fin, dh, G + st->po.W1, T, H, F);
    const void* da;     // gradient at the attention block's output
    if (c.arch == BAMBOO_ARCH_POST_LN_ENCODER) {
      d = gemm_nt(dh, P(st->po.W1), d2, T, H, F, EPI_RES);   // + residual branch of r2 = y1 + f
      d.res = df;
      BBCHK(p_gemm(st, s, K_DGRAD_FFN1, d));
      BBCHK(p_ln_bwd(st, s, ws, T, H, d2, rec + r.r1, (const float*)(rec + r.ln1), P(st->po.g1), nullptr, d1,
                     G + st->po.g1, G + st->po.be1, G + st->po.bo, w.p_ln[0], &batch));
      da = d1;
    } else {
      BBCHK(p_gemm(st, s, K_DGRAD_FFN1, gemm_nt(dh, P(st->po.W1), d1, T, H, F, EPI_STORE)));
      BBCHK(p_ln_bwd(st, s, ws, T, H, d1, rec + r.r1, (const float*)(rec + r.ln2), P(st->po.g2), dy, d2,
                     G + st->po.g2, G + st->po.be2, G + st->po.bo, w.p_ln[1], &batch));   // + residual branch of y = x1 + f
      da = d2;
    }
    // a = ctx Wo + bo
    wgrad[2] = gemm_tn(rec + r.ctx, da, G + st->po.Wo, T, H, H);
    BBCHK(p_gemm(st, s, K_DGRAD_ATTN_OUT, gemm_nt(da, P(st->po.Wo), dctx, T, H, H, EPI_STORE)));
    // the MFMA kernels also leave the column sums of dqkv (the gradient of bqkv), one partial row per sample
    // and block of 128 tokens; any other kernel leaves dqkv_parts at 0 and a column-sum launch follows
    int dqkv_parts = 0;
    if ((size_t)c.micro_batch * ((c.seq + 127) / 128) <= reduce_max_partials()) {
      a.dqkv_colsum = (float*)(ws + w.p_dqkv);
      a.dqkv_colsum_parts = &dqkv_parts;
    }
    BBCHK(p_attn_bwd(st, s, a));
    // qkv = ain Wqkv + bqkv
    if (dqkv_parts > 0) {
      if (!grad_reduce_add(&batch, 3 * H, dqkv_parts, (const float*)(ws + w.p_dqkv), G + st->po.bqkv, nullptr, nullptr))
        return BAMBOO_E_STATE;
    } else {
      BBCHK(p_colsum(st, s, ws, T, 3 * H, dqkv, G + st->po.bqkv, w.p_dqkv, &batch));
    }
    wgrad[3] = gemm_tn(rec + r.ain, dqkv, G + st->po.Wqkv, T, H, 3 * H);
    if (c.arch == BAMBOO_ARCH_POST_LN_ENCODER) {
      d = gemm_nt(dqkv, P(st->po.Wqkv), dx, T, H, 3 * H, EPI_RES);   // + residual branch of r1 = x + a
      d.res = da;
      BBCHK(p_gemm(st, s, K_DGRAD_QKV, d));
    } else {
      BBCHK(p_gemm(st, s, K_DGRAD_QKV, gemm_nt(dqkv, P(st->po.Wqkv), d1, T, H, 3 * H, EPI_STORE)));
      BBCHK(p_ln_bwd(st, s, ws, T, H, d1, rec + r.x, (const float*)(rec + r.ln1), P(st->po.g1), da, dx,
                     G + st->po.g1, G + st->po.be1, nullptr, w.p_ln[0], &batch));   // + residual branch of x1 = x + a
    }
    // The ordered final sums of the layer's partial rows ride in the weight-gradient launch where the
    // grouped MFMA kernel runs it (its last tiles leave CUs idle); otherwise a launch of their own.
    bool reduced = false;
    BBCHK(p_gemm_group(st, s, wgrad, 4, &batch, &reduced));
    if (!reduced) BBCHK(p_grad_reduce(st, s, batch));
    dy = dx;
  }
  return BAMBOO_OK;
}

bool swapping(const bamboo_stage* st) { return st->cfg.swap_slots > 0; }
uint64_t shadow_slot_bytes(const bamboo_stage* st) { return (uint64_t)st->cfg.n_shadow * st->rl.bytes; }

// Copy host_stash[k] back into ring slot k mod R on the swap stream.  The copy waits for the
// last reader of the slot; a writer of the slot (FRC) and its copy out precede it in the swap
// stream's own order.
int swap_in(bamboo_stage* st, int k) {
  const int d = k % st->cfg.swap_slots;
  const uint64_t nb = shadow_slot_bytes(st);
  HIPCHK(hipStreamWaitEvent(st->lane_swap, st->ev_read[d], 0));
  HIPCHK(hipMemcpyAsync(st->stash[1] + (uint64_t)d * nb, st->host_stash + (uint64_t)k * nb, nb, hipMemcpyHostToDevice,
                        st->lane_swap));
  HIPCHK(hipEventRecord(st->ev_in[d], st->lane_swap));
  st->ring_mb[d] = k;
  return BAMBOO_OK;
}

// The micro-batch of the first BRC after BRC(k) in the stage's current program, or -1.
int next_brc_after(const bamboo_stage* st, int k) {
  const std::vector<bamboo_instr_t>& p = st->program;
  size_t i = 0;
  while (i < p.size() && !(p[i].op == BAMBOO_BRC && p[i].mb == k)) ++i;
  for (++i; i < p.size(); ++i)
    if (p[i].op == BAMBOO_BRC) return p[i].mb;
  return -1;
}

int get_event(std::vector<hipEvent_t>& v, int k, hipEvent_t* out) {
  if (v[k] == nullptr) HIPCHK(hipEventCreateWithFlags(&v[k], hipEventDisableTiming));
  *out = v[k];
  return BAMBOO_OK;
}

}  // namespace

extern "C" {

const char* stage_strerror(int status) {
  switch (status) {
    case BAMBOO_OK: return "ok";
    case BAMBOO_E_BADCFG: return "configuration rejected";
    case BAMBOO_E_BADMB: return "micro-batch id out of range or no stashed forward for it";
    case BAMBOO_E_STATE: return "call not valid in the stage's current state";
    case BAMBOO_E_HIP: return "HIP runtime call failed";
    case BAMBOO_E_ARG: return "bad argument (null pointer, small buffer or misaligned pointer)";
    case BAMBOO_E_NOMEM: return "host allocation failed";
    default: return "unknown status";
  }
}

int stage_query_sizes(const bamboo_cfg_t* cfg, bamboo_sizes_t* out) {
  const int v = validate(cfg);
  if (v != BAMBOO_OK) return v;
  if (!out) return BAMBOO_E_ARG;
  const uint64_t es = cfg->dtype == BAMBOO_BF16 ? 2 : 4;
  const ParamOffsets po = param_offsets(cfg->hidden, cfg->ffn);
  const RecordLayout rl = record_layout(*cfg);
  memset(out, 0, sizeof(*out));
  out->layer_params = po.count;
  out->own_w = po.count * cfg->n_own * es;
  out->shadow_w = po.count * cfg->n_shadow * es;
  out->own_g = po.count * cfg->n_own * 4;
  out->shadow_g = po.count * cfg->n_shadow * 4;
  out->rec_bytes = rl.bytes;
  out->c_own = own_slot_count(cfg->P, cfg->stage_id, cfg->M);
  out->c_shadow = cfg->n_shadow > 0 ? (cfg->swap_slots > 0 ? cfg->swap_slots : cfg->M) : 0;
  out->host_stash = cfg->swap_slots > 0 ? (uint64_t)cfg->M * cfg->n_shadow * rl.bytes : 0;
  out->own_stash = (uint64_t)out->c_own * cfg->n_own * rl.bytes;
  out->shadow_stash = (uint64_t)out->c_shadow * cfg->n_shadow * rl.bytes;
  out->workspace = lane_scratch(*cfg, true).bytes + lane_scratch(*cfg, cfg->rc_mode == BAMBOO_RC_EFEB).bytes;
  out->own_opt = po.count * cfg->n_own * 12;
  out->shadow_opt = po.count * cfg->n_shadow * 12;
  return BAMBOO_OK;
}

int stage_program(const bamboo_cfg_t* cfg, bamboo_instr_t* out, int32_t cap) {
  const int v = validate(cfg);
  if (v != BAMBOO_OK) return v;
  try {
    return copy_out(build_program(*cfg), out, cap);
  } catch (const std::bad_alloc&) {
    return BAMBOO_E_NOMEM;
  }
}

int stage_program_uneven(const bamboo_cfg_t* cfg, const int32_t* tick_F, const int32_t* tick_B, bamboo_instr_t* out,
                         int32_t cap) {
  const int v = validate(cfg);
  if (v != BAMBOO_OK) return v;
  for (int st = 0; st < cfg->P; ++st)
    if ((tick_F && tick_F[st] < 1) || (tick_B && tick_B[st] < 1)) return BAMBOO_E_BADCFG;
  try {
    return copy_out(build_program(*cfg, tick_F, tick_B), out, cap);
  } catch (const std::bad_alloc&) {
    return BAMBOO_E_NOMEM;
  }
}

int stage_failover_program(const bamboo_cfg_t* cfg, int32_t k_fail, bamboo_instr_t* out, int32_t cap) {
  const int v = validate(cfg);
  if (v != BAMBOO_OK) return v;
  if (!can_fail_over(*cfg)) return BAMBOO_E_STATE;
  if (k_fail < 0 || k_fail >= cfg->M) return BAMBOO_E_BADMB;
  try {
    return copy_out(failover_list(*cfg, k_fail), out, cap);
  } catch (const std::bad_alloc&) {
    return BAMBOO_E_NOMEM;
  }
}

int stage_merged_program(const bamboo_cfg_t* cfg, bamboo_instr_t* out, int32_t cap) {
  const int v = validate(cfg);
  if (v != BAMBOO_OK) return v;
  if (!can_fail_over(*cfg)) return BAMBOO_E_STATE;
  try {
    return copy_out(merged_list(*cfg), out, cap);
  } catch (const std::bad_alloc&) {
    return BAMBOO_E_NOMEM;
  }
}

int stage_wrap_victim_progress(const bamboo_cfg_t* cfg, int32_t k_fail, int32_t* n_fwd, int32_t* n_bwd) {
  const int v = validate(cfg);
  if (v != BAMBOO_OK) return v;
  if (!n_fwd || !n_bwd) return BAMBOO_E_ARG;
  if (!cfg->wrap) return BAMBOO_E_STATE;
  if (k_fail < 0 || k_fail >= cfg->M) return BAMBOO_E_BADMB;
  try {
    int a = 0, b = 0;
    wrap_victim_progress(*cfg, k_fail, &a, &b);
    *n_fwd = a;
    *n_bwd = b;
  } catch (const std::bad_alloc&) {
    return BAMBOO_E_NOMEM;
  }
  return BAMBOO_OK;
}

int64_t stage_record_offset(const bamboo_cfg_t* cfg, int32_t kind, int32_t slot, int32_t layer) {
  bamboo_sizes_t sz;
  const int v = stage_query_sizes(cfg, &sz);
  if (v != BAMBOO_OK) return v;
  const int n = kind == 0 ? cfg->n_own : cfg->n_shadow;
  const int slots = kind == 0 ? sz.c_own : sz.c_shadow;
  if ((kind != 0 && kind != 1) || slot < 0 || slot >= slots || layer < 0 || layer >= n) return BAMBOO_E_ARG;
  return (int64_t)(((uint64_t)slot * n + layer) * sz.rec_bytes);
}

int stage_record_fields(const bamboo_cfg_t* cfg, uint64_t out[13]) {
  const int v = validate(cfg);
  if (v != BAMBOO_OK) return v;
  if (!out) return BAMBOO_E_ARG;
  const RecordLayout r = record_layout(*cfg);
  const uint64_t f[13] = {r.x, r.ain, r.qkv, r.ctx, r.r1, r.fin, r.g, r.dg, r.r2, r.lse, r.ln1, r.ln2, r.bytes};
  memcpy(out, f, sizeof(f));
  return BAMBOO_OK;
}

int stage_workspace_fields(const bamboo_cfg_t* cfg, uint64_t out[7]) {
  const int v = validate(cfg);
  if (v != BAMBOO_OK) return v;
  if (!out) return BAMBOO_E_ARG;
  const LaneScratch w = lane_scratch(*cfg, true);
  const uint64_t f[7] = {w.dh, w.d1, w.d2, w.d3, w.dctx, w.dqkv, w.bytes};
  memcpy(out, f, sizeof(f));
  return BAMBOO_OK;
}

int stage_init(const bamboo_cfg_t* cfg, const bamboo_sizes_t* sizes, const void* own_w, const void* shadow_w,
               void* own_g, void* shadow_g, void* own_stash, void* shadow_stash, void* workspace, void* stream_main,
               void* stream_frc, bamboo_stage_t** out) {
  bamboo_sizes_t need;
  const int v = stage_query_sizes(cfg, &need);
  if (v != BAMBOO_OK) return v;
  if (!sizes || !out || !own_w || !own_g || !own_stash || !workspace) return BAMBOO_E_ARG;
  if (cfg->n_shadow > 0 && (!shadow_w || !shadow_g || !shadow_stash)) return BAMBOO_E_ARG;
  if (sizes->own_w < need.own_w || sizes->shadow_w < need.shadow_w || sizes->own_g < need.own_g ||
      sizes->shadow_g < need.shadow_g || sizes->own_stash < need.own_stash ||
      sizes->shadow_stash < need.shadow_stash || sizes->workspace < need.workspace)
    return BAMBOO_E_ARG;
  const void* ptrs[] = {own_w, shadow_w, own_g, shadow_g, own_stash, shadow_stash, workspace};
  for (const void* p : ptrs)
    if (((uintptr_t)p) % kAlign) return BAMBOO_E_ARG;
  bamboo_stage* st = new (std::nothrow) bamboo_stage();
  if (!st) return BAMBOO_E_NOMEM;
  try {
    st->cfg = *cfg;
    st->sizes = need;
    st->po = param_offsets(cfg->hidden, cfg->ffn);
    st->rl = record_layout(*cfg);
    st->ws0 = lane_scratch(*cfg, true);
    st->ws1 = lane_scratch(*cfg, cfg->rc_mode == BAMBOO_RC_EFEB);   // lane 1 runs backwards only with eager BRC
    st->w[0] = (const char*)own_w;
    st->w[1] = (const char*)shadow_w;
    st->g[0] = (float*)own_g;
    st->g[1] = (float*)shadow_g;
    st->stash[0] = (char*)own_stash;
    st->stash[1] = (char*)shadow_stash;
    st->wsbase = (char*)workspace;
    st->lane[0] = (hipStream_t)stream_main;
    st->lane[1] = (hipStream_t)stream_frc;
    st->program = build_program(*cfg);
    st->merged = false;
    st->own_slot_mb.assign(need.c_own, -1);
    st->fwd_issued.assign(cfg->M, 0);
    st->frc_issued.assign(cfg->M, 0);
    st->shadow_live.assign(cfg->M, 0);
    st->bwd_done.assign(cfg->M, 0);
    st->merged_program_installed = false;
    st->apply_step = 0;
    st->ev_fwd.assign(cfg->M, nullptr);
    st->ev_frc.assign(cfg->M, nullptr);
    st->ev_join = nullptr;
    st->last_frc_on_lane1 = -1;
    st->prof_on = false;
    st->opt[0] = st->opt[1] = nullptr;
    st->host_stash = nullptr;
    st->lane_swap = nullptr;
    st->ev_swap_join = nullptr;
    st->on_host.assign(cfg->M, 0);
  } catch (const std::bad_alloc&) {
    delete st;
    return BAMBOO_E_NOMEM;
  }
  if (cfg->dtype == BAMBOO_BF16 && prepare_gemm_tables((hipStream_t)stream_main) != hipSuccess) {
    (void)hipGetLastError();
    delete st;
    return BAMBOO_E_HIP;
  }
  if (hipEventCreateWithFlags(&st->ev_join, hipEventDisableTiming) != hipSuccess) {
    (void)hipGetLastError();
    delete st;
    return BAMBOO_E_HIP;
  }
  *out = st;
  return BAMBOO_OK;
}

int stage_schedule(const bamboo_stage_t* st, bamboo_instr_t* out, int32_t cap) {
  if (!st) return BAMBOO_E_ARG;
  return copy_out(st->program, out, cap);
}

int stage_begin_iteration(bamboo_stage_t* st) {
  if (!st) return BAMBOO_E_ARG;
  std::fill(st->own_slot_mb.begin(), st->own_slot_mb.end(), -1);
  std::fill(st->fwd_issued.begin(), st->fwd_issued.end(), 0);
  std::fill(st->frc_issued.begin(), st->frc_issued.end(), 0);
  std::fill(st->shadow_live.begin(), st->shadow_live.end(), 0);
  std::fill(st->bwd_done.begin(), st->bwd_done.end(), 0);
  // the first iteration after a merge: the failover list (which starts in mid-iteration) gives way to
  // the merged stage's whole-iteration program
  if (st->merged && !st->merged_program_installed) {
    try {
      st->program = merged_list(st->cfg);
    } catch (const std::bad_alloc&) {
      return BAMBOO_E_NOMEM;
    }
    st->merged_program_installed = true;
  }
  std::fill(st->ring_mb.begin(), st->ring_mb.end(), -1);
  std::fill(st->on_host.begin(), st->on_host.end(), 0);
  st->last_frc_on_lane1 = -1;
  return BAMBOO_OK;
}

int stage_fwd(bamboo_stage_t* st, int32_t k, const void* x, void* y) {
  if (!st || !x || !y) return BAMBOO_E_ARG;
  if (k < 0 || k >= st->cfg.M) return BAMBOO_E_BADMB;
  const int slot = k % st->sizes.c_own;
  if (st->own_slot_mb[slot] != -1 || st->fwd_issued[k]) return BAMBOO_E_BADMB;
  const int rc = run_forward(st, 0, 0, slot, x, y);
  if (rc != BAMBOO_OK) return rc;
  st->own_slot_mb[slot] = k;
  st->fwd_issued[k] = 1;
  hipEvent_t ev;
  if (get_event(st->ev_fwd, k, &ev) != BAMBOO_OK) return BAMBOO_E_HIP;
  HIPCHK(hipEventRecord(ev, st->lane[0]));
  return BAMBOO_OK;
}

int shadow_fwd_frc(bamboo_stage_t* st, int32_t k, const void* y, void* z) {
  if (!st || !y) return BAMBOO_E_ARG;
  // lazy FRC: only the failover schedule runs it
  if (st->cfg.n_shadow <= 0 || (st->cfg.rc_mode == BAMBOO_RC_LFLB && !st->merged)) return BAMBOO_E_STATE;
  if (k < 0 || k >= st->cfg.M) return BAMBOO_E_BADMB;
  // the replica of the first stage works on the samples, the replica of a data-parallel peer on that
  // peer's minibatch: not on this stage's output
  const bool input_is_own_output = !st->cfg.wrap && !st->cfg.data_parallel;
  if ((!st->fwd_issued[k] && input_is_own_output) || st->frc_issued[k]) return BAMBOO_E_BADMB;
  const int lane_id = st->merged ? 0 : 1;
  hipEvent_t ev;
  if (lane_id == 1 && input_is_own_output) {
    if (get_event(st->ev_fwd, k, &ev) != BAMBOO_OK) return BAMBOO_E_HIP;
    HIPCHK(hipStreamWaitEvent(st->lane[1], ev, 0));
  }
  char* ws = st->wsbase + (lane_id == 0 ? 0 : st->ws0.bytes);
  void* zout = z ? z : (void*)(ws + (lane_id == 0 ? st->ws0.out : st->ws1.out));
  int slot = k;
  if (swapping(st)) {
    if (!st->host_stash) return BAMBOO_E_STATE;
    // the ring slot may be overwritten once its last occupant is on the host, no copy into it is
    // in flight and its last reader is done
    slot = k % st->cfg.swap_slots;
    HIPCHK(hipStreamWaitEvent(st->lane[lane_id], st->ev_out[slot], 0));
    HIPCHK(hipStreamWaitEvent(st->lane[lane_id], st->ev_in[slot], 0));
    HIPCHK(hipStreamWaitEvent(st->lane[lane_id], st->ev_read[slot], 0));
  }
  const int rc = run_forward(st, 1, lane_id, slot, y, zout);
  if (rc != BAMBOO_OK) return rc;
  st->frc_issued[k] = 1;
  st->shadow_live[k] = 1;
  if (swapping(st)) {
    const uint64_t nb = shadow_slot_bytes(st);
    HIPCHK(hipEventRecord(st->ev_written[slot], st->lane[lane_id]));
    HIPCHK(hipStreamWaitEvent(st->lane_swap, st->ev_written[slot], 0));
    HIPCHK(hipMemcpyAsync(st->host_stash + (uint64_t)k * nb, st->stash[1] + (uint64_t)slot * nb, nb,
                          hipMemcpyDeviceToHost, st->lane_swap));
    HIPCHK(hipEventRecord(st->ev_out[slot], st->lane_swap));
    st->ring_mb[slot] = k;
    st->on_host[k] = 1;
  }
  if (lane_id == 1) {
    if (get_event(st->ev_frc, k, &ev) != BAMBOO_OK) return BAMBOO_E_HIP;
    HIPCHK(hipEventRecord(ev, st->lane[1]));
    st->last_frc_on_lane1 = k;
  }
  return BAMBOO_OK;
}

int stage_bwd(bamboo_stage_t* st, int32_t k, const void* gy, void* gx) {
  if (!st || !gy || !gx) return BAMBOO_E_ARG;
  if (k < 0 || k >= st->cfg.M) return BAMBOO_E_BADMB;
  const int slot = k % st->sizes.c_own;
  if (st->own_slot_mb[slot] != k) return BAMBOO_E_BADMB;
  const int rc = run_backward(st, 0, 0, slot, gy, gx);
  if (rc != BAMBOO_OK) return rc;
  st->own_slot_mb[slot] = -1;
  st->bwd_done[k] = 1;
  return BAMBOO_OK;
}

int shadow_bwd_brc(bamboo_stage_t* st, int32_t k, const void* gz, void* gy) {
  if (!st || !gz) return BAMBOO_E_ARG;
  // lazy BRC runs after a preemption only; eager BRC (EFEB) also before, on the FRC lane
  if (st->cfg.n_shadow <= 0 || (!st->merged && st->cfg.rc_mode != BAMBOO_RC_EFEB)) return BAMBOO_E_STATE;
  if (k < 0 || k >= st->cfg.M) return BAMBOO_E_BADMB;
  if (!st->shadow_live[k]) return BAMBOO_E_STATE;
  const int lane_id = st->merged ? 0 : 1;
  // on lane 1 BRC(k) follows FRC(k) in stream order; on lane 0 it waits for an FRC issued on lane 1
  if (lane_id == 0 && st->ev_frc[k] != nullptr) HIPCHK(hipStreamWaitEvent(st->lane[0], st->ev_frc[k], 0));
  int slot = k;
  if (swapping(st)) {
    if (!st->host_stash || !st->on_host[k]) return BAMBOO_E_STATE;
    slot = k % st->cfg.swap_slots;
    if (st->ring_mb[slot] != k) {
      const int e = swap_in(st, k);
      if (e != BAMBOO_OK) return e;
    }
    HIPCHK(hipStreamWaitEvent(st->lane[lane_id], st->ev_written[slot], 0));
    HIPCHK(hipStreamWaitEvent(st->lane[lane_id], st->ev_in[slot], 0));
  }
  const int rc = run_backward(st, 1, lane_id, slot, gz, gy);
  if (rc != BAMBOO_OK) return rc;
  st->shadow_live[k] = 0;
  if (swapping(st)) {
    HIPCHK(hipEventRecord(st->ev_read[slot], st->lane[lane_id]));
    st->ring_mb[slot] = -1;     // consumed: nothing to keep
    // start bringing in what the next BRC needs while this one runs
    const int k2 = next_brc_after(st, k);
    if (k2 >= 0 && k2 < st->cfg.M && st->on_host[k2] && st->shadow_live[k2]) {
      const int d2 = k2 % st->cfg.swap_slots;
      if (d2 != slot && st->ring_mb[d2] != k2) {
        const int e = swap_in(st, k2);
        if (e != BAMBOO_OK) return e;
      }
    }
  }
  return BAMBOO_OK;
}

int failover_merge(bamboo_stage_t* st, int32_t k_fail, bamboo_instr_t* out, int32_t cap) {
  if (!st) return BAMBOO_E_ARG;
  if (st->merged || !can_fail_over(st->cfg)) return BAMBOO_E_STATE;
  if (k_fail < 0 || k_fail >= st->cfg.M) return BAMBOO_E_BADMB;
  std::vector<bamboo_instr_t> prog;
  try {
    prog = failover_list(st->cfg, k_fail);
  } catch (const std::bad_alloc&) {
    return BAMBOO_E_NOMEM;
  }
  // the size-query form (NULL, 0) of the other schedule calls would merge the stage for good: rejected
  if (out == nullptr) return BAMBOO_E_ARG;
  const int n = copy_out(prog, out, cap);
  if (n < 0) return n;
  // JOIN: everything issued on the FRC lane must be visible to lane 0
  HIPCHK(hipEventRecord(st->ev_join, st->lane[1]));
  HIPCHK(hipStreamWaitEvent(st->lane[0], st->ev_join, 0));
  st->merged = true;
  st->program.swap(prog);
  return n;
}

int stage_run(bamboo_stage_t* st, const bamboo_instr_t* program, int32_t n, const bamboo_tables_t* t) {
  if (!st || !t || n < 0 || (n > 0 && !program)) return BAMBOO_E_ARG;
  // an instruction of the wrap-around stage is a pair of calls into two objects (the stage and the
  // model's ends): the caller composes them
  if (st->cfg.wrap) return BAMBOO_E_STATE;
  const int M = st->cfg.M;
  for (int32_t i = 0; i < n; ++i) {
    const bamboo_instr_t& in = program[i];
    const int k = in.mb;
    const bool needs_mb = in.op == BAMBOO_FWD || in.op == BAMBOO_BWD || in.op == BAMBOO_FRC || in.op == BAMBOO_BRC;
    if (needs_mb && (k < 0 || k >= M)) return BAMBOO_E_BADMB;
    int rc = BAMBOO_OK;
    switch (in.op) {
      case BAMBOO_FWD:
        if (!t->x || !t->y) return BAMBOO_E_ARG;
        rc = stage_fwd(st, k, t->x[k], t->y[k]);
        break;
      case BAMBOO_FRC: {
        const void* src = t->frc_in ? t->frc_in[k] : (t->y ? t->y[k] : nullptr);
        if (!src) return BAMBOO_E_ARG;
        rc = shadow_fwd_frc(st, k, src, t->z ? t->z[k] : nullptr);
        break;
      }
      case BAMBOO_BWD:
        if (!t->gy || !t->gx) return BAMBOO_E_ARG;
        rc = stage_bwd(st, k, t->gy[k], t->gx[k]);
        break;
      case BAMBOO_BRC:
        if (!t->gz) return BAMBOO_E_ARG;
        if (!st->merged) {
          rc = shadow_bwd_brc(st, k, t->gz[k], nullptr);     // beside a live successor: its g_y is the successor's to deliver
        } else if (st->bwd_done[k] || st->cfg.data_parallel) {
          // replayed, or a data-parallel peer's input gradient: it feeds nothing on this node
          rc = shadow_bwd_brc(st, k, t->gz[k], t->gy_replay ? t->gy_replay[k] : nullptr);
        } else {
          if (!t->gy) return BAMBOO_E_ARG;
          rc = shadow_bwd_brc(st, k, t->gz[k], t->gy[k]);   // the gradient the victim would have sent: feeds BWD(k)
        }
        break;
      case BAMBOO_BUBBLE:
        if (t->us_per_tick > 0.f) rc = stage_bubble(st, in.arg, t->us_per_tick);
        break;
      case BAMBOO_JOIN:
        rc = stage_join(st);
        break;
      case BAMBOO_APPLY:
        if (t->adam && st->opt[0]) rc = stage_apply(st, t->adam, ++st->apply_step);
        break;
      case BAMBOO_RECV_ACT:
      case BAMBOO_SEND_ACT:
      case BAMBOO_RECV_GRAD:
      case BAMBOO_SEND_GRAD:
      case BAMBOO_ALLREDUCE:
        if (t->comm && t->comm(t->user, &in) != 0) return i;   // the peer is gone: the caller fails over
        break;
      default:
        return BAMBOO_E_ARG;
    }
    if (rc != BAMBOO_OK) return rc;
  }
  return n;
}

int stage_optimizer_init(bamboo_stage_t* st, void* own_opt, void* shadow_opt) {
  if (!st || !own_opt) return BAMBOO_E_ARG;
  if (st->cfg.n_shadow > 0 && !shadow_opt) return BAMBOO_E_ARG;
  if (((uintptr_t)own_opt) % kAlign || ((uintptr_t)shadow_opt) % kAlign) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  void* bufs[2] = {own_opt, st->cfg.n_shadow > 0 ? shadow_opt : nullptr};
  for (int kind = 0; kind < 2; ++kind) {
    st->opt[kind] = (float*)bufs[kind];
    if (!bufs[kind]) continue;
    const long n = (long)st->po.count * (kind == 0 ? st->cfg.n_own : st->cfg.n_shadow);
    HIPCHK(launch_widen(st->lane[0], st->cfg.dtype, n, st->w[kind], st->opt[kind]));
    HIPCHK(launch_fill_zero(st->lane[0], 2 * n, st->opt[kind] + n));
  }
  return BAMBOO_OK;
}

int stage_apply(bamboo_stage_t* st, const bamboo_adam_t* hp, int32_t step) {
  if (!st || !hp) return BAMBOO_E_ARG;
  if (step < 1 || !(hp->lr >= 0.f) || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) ||
      !(hp->eps > 0.f))
    return BAMBOO_E_ARG;
  if (!st->opt[0]) return BAMBOO_E_STATE;
  (void)hipGetLastError();
  const int kinds = st->merged ? 2 : 1;     // the merged stage owns the victim's layers too
  for (int kind = 0; kind < kinds; ++kind) {
    if (!st->opt[kind]) return BAMBOO_E_STATE;
    const long n = (long)st->po.count * (kind == 0 ? st->cfg.n_own : st->cfg.n_shadow);
    float* o = st->opt[kind];
    HIPCHK(launch_adam(st->lane[0], st->cfg.dtype, n, st->g[kind], o, o + n, o + 2 * n, (void*)st->w[kind], hp->lr,
                       hp->beta1, hp->beta2, hp->eps, step));
  }
  return BAMBOO_OK;
}

int stage_sync_replica(bamboo_stage_t* st, const void* successor_w, const void* successor_opt) {
  if (!st || !successor_w) return BAMBOO_E_ARG;
  if (st->cfg.n_shadow <= 0 || st->merged) return BAMBOO_E_STATE;   // no replica / the victim is gone
  if (successor_opt && !st->opt[1]) return BAMBOO_E_STATE;
  (void)hipGetLastError();
  // lane 1 may still be reading the replica parameters (FRC of the iteration that just ended)
  HIPCHK(hipEventRecord(st->ev_join, st->lane[1]));
  HIPCHK(hipStreamWaitEvent(st->lane[0], st->ev_join, 0));
  HIPCHK(launch_copy(st->lane[0], successor_w, (void*)st->w[1], st->sizes.shadow_w));
  if (successor_opt) HIPCHK(launch_copy(st->lane[0], successor_opt, st->opt[1], st->sizes.shadow_opt));
  // and the next iteration's FRC on lane 1 must see the new values
  HIPCHK(hipEventRecord(st->ev_join, st->lane[0]));
  HIPCHK(hipStreamWaitEvent(st->lane[1], st->ev_join, 0));
  return BAMBOO_OK;
}

int stage_bubble(bamboo_stage_t* st, int32_t ticks, float us_per_tick) {
  if (!st) return BAMBOO_E_ARG;
  if (ticks < 0 || !(us_per_tick >= 0.f)) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  HIPCHK(launch_bubble(st->lane[0], (float)ticks * us_per_tick));
  return BAMBOO_OK;
}

int stage_join(bamboo_stage_t* st) {
  if (!st) return BAMBOO_E_ARG;
  HIPCHK(hipEventRecord(st->ev_join, st->lane[1]));
  HIPCHK(hipStreamWaitEvent(st->lane[0], st->ev_join, 0));
  if (st->host_stash) {
    HIPCHK(hipEventRecord(st->ev_swap_join, st->lane_swap));
    HIPCHK(hipStreamWaitEvent(st->lane[0], st->ev_swap_join, 0));
  }
  return BAMBOO_OK;
}

int stage_sync(bamboo_stage_t* st) {
  const int rc = stage_join(st);
  if (rc != BAMBOO_OK) return rc;
  HIPCHK(hipStreamSynchronize(st->lane[0]));
  HIPCHK(hipStreamSynchronize(st->lane[1]));
  if (st->host_stash) HIPCHK(hipStreamSynchronize(st->lane_swap));
  return BAMBOO_OK;
}

int stage_swap_attach(bamboo_stage_t* st, void* host_stash, uint64_t bytes, void* stream_swap) {
  if (!st || !host_stash) return BAMBOO_E_ARG;
  if (!swapping(st) || st->host_stash) return BAMBOO_E_STATE;
  if (bytes < st->sizes.host_stash || ((uintptr_t)host_stash % 16)) return BAMBOO_E_ARG;
  const int R = st->cfg.swap_slots;
  std::vector<hipEvent_t> ev;
  try {
    ev.assign(4 * (size_t)R + 1, nullptr);
    st->ring_mb.assign(R, -1);
    st->ev_written.resize(R); st->ev_out.resize(R); st->ev_in.resize(R); st->ev_read.resize(R);
  } catch (const std::bad_alloc&) {
    return BAMBOO_E_NOMEM;
  }
  for (size_t i = 0; i < ev.size(); ++i)
    if (hipEventCreateWithFlags(&ev[i], hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
      st->ring_mb.clear(); st->ev_written.clear(); st->ev_out.clear(); st->ev_in.clear(); st->ev_read.clear();
      return BAMBOO_E_HIP;
    }
  for (int d = 0; d < R; ++d) {
    st->ev_written[d] = ev[4 * d]; st->ev_out[d] = ev[4 * d + 1]; st->ev_in[d] = ev[4 * d + 2]; st->ev_read[d] = ev[4 * d + 3];
  }
  st->ev_swap_join = ev[4 * (size_t)R];
  st->lane_swap = (hipStream_t)stream_swap;
  st->host_stash = (char*)host_stash;
  return BAMBOO_OK;
}

int stage_profile(bamboo_stage_t* st, int enable) {
  if (!st) return BAMBOO_E_ARG;
  for (auto& r : st->prof_recs) {
    st->prof_pool.push_back(r.a);
    st->prof_pool.push_back(r.b);
  }
  st->prof_recs.clear();
  st->prof_on = enable != 0;
  return BAMBOO_OK;
}

int stage_profile_read(bamboo_stage_t* st, int32_t kernel_class, double* total_ms, int64_t* launches, double* work) {
  if (!st || !total_ms || !launches || !work) return BAMBOO_E_ARG;
  if (kernel_class < 0 || kernel_class >= K_COUNT) return BAMBOO_E_ARG;
  const int rc = stage_sync(st);
  if (rc != BAMBOO_OK) return rc;
  double ms = 0.0, w = 0.0;
  int64_t n = 0;
  for (auto& r : st->prof_recs) {
    if (r.cls != kernel_class) continue;
    float t = 0.f;
    HIPCHK(hipEventElapsedTime(&t, r.a, r.b));
    ms += t;
    w += r.work;
    ++n;
  }
  *total_ms = ms;
  *launches = n;
  *work = w;
  return BAMBOO_OK;
}

int stage_destroy(bamboo_stage_t* st) {
  if (!st) return BAMBOO_E_ARG;
  for (auto& r : st->prof_recs) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  for (hipEvent_t e : st->prof_pool) (void)hipEventDestroy(e);
  for (hipEvent_t e : st->ev_fwd)
    if (e) (void)hipEventDestroy(e);
  for (hipEvent_t e : st->ev_frc)
    if (e) (void)hipEventDestroy(e);
  if (st->ev_join) (void)hipEventDestroy(st->ev_join);
  for (auto* v : {&st->ev_written, &st->ev_out, &st->ev_in, &st->ev_read})
    for (hipEvent_t e : *v)
      if (e) (void)hipEventDestroy(e);
  if (st->ev_swap_join) (void)hipEventDestroy(st->ev_swap_join);
  delete st;
  return BAMBOO_OK;
}

}  // extern "C"
