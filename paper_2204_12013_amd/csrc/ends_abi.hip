// The two ends of the model around a wrap-around stage: buffer layout and launch
// order only; the arithmetic is in ends.hip, the GEMM and LayerNorm kernels.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <vector>

#include "../../include/bamboo_ends.h"
#include "common.h"

using namespace bamboo;

namespace {
constexpr uint64_t kAlign = 256;
inline uint64_t up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct EndsLayout {
  uint64_t es;
  // parameter offsets in elements
  uint64_t f_tok, f_pos, f_g, f_b, front_params;
  uint64_t b_g, b_b, b_head, back_params;
  // front stash slot
  uint64_t fs_ids, fs_e, fs_stats, fs_bytes;
  // back stash
  uint64_t bs_y, bs_stats, bs_hf, bs_logits, bs_lse, bs_tok, bs_labels, bs_bytes;
  // workspace
  uint64_t ws_d, ws_partial, ws_bytes;
};

EndsLayout layout(const bamboo_cfg_t& c, int V) {
  EndsLayout l;
  memset(&l, 0, sizeof(l));
  const uint64_t T = (uint64_t)c.micro_batch * c.seq, H = c.hidden, S = c.seq;
  const bool enc = c.arch == BAMBOO_ARCH_POST_LN_ENCODER;
  l.es = c.dtype == BAMBOO_BF16 ? 2 : 4;
  l.f_tok = 0; l.f_pos = (uint64_t)V * H; l.f_g = l.f_pos + S * H; l.f_b = l.f_g + H;
  l.front_params = l.f_g + (enc ? 2 * H : 0);
  l.b_g = 0; l.b_b = H; l.b_head = enc ? 0 : 2 * H;
  l.back_params = l.b_head + H * (uint64_t)V;
  uint64_t o = 0;
  l.fs_ids = o; o += up(T * 4);
  l.fs_e = o; o += enc ? up(T * H * l.es) : 0;
  l.fs_stats = o; o += enc ? up(T * 8) : 0;
  l.fs_bytes = o;
  o = 0;
  l.bs_y = o; o += up(T * H * l.es);
  l.bs_stats = o; o += enc ? 0 : up(T * 8);
  l.bs_hf = o; o += enc ? 0 : up(T * H * l.es);
  l.bs_logits = o; o += up(T * (uint64_t)V * l.es);
  l.bs_lse = o; o += up(T * 4);
  l.bs_tok = o; o += up(T * 4);
  l.bs_labels = o; o += up(T * 4);
  l.bs_bytes = o;
  o = 0;
  l.ws_d = o; o += up(T * H * l.es);
  l.ws_partial = o; o += up(ln_bwd_partial_floats((int)H) * 4);
  l.ws_bytes = o;
  return l;
}

int check_cfg(const bamboo_cfg_t* cfg, int32_t vocab) {
  bamboo_sizes_t sz;
  const int v = stage_query_sizes(cfg, &sz);   // the stage's own validation
  if (v != BAMBOO_OK) return v;
  if (vocab <= 0 || vocab % 8) return BAMBOO_E_BADCFG;
  return BAMBOO_OK;
}

#define ENDCHK(expr)                                                                                      \
  do {                                                                                                    \
    const hipError_t e_ = (expr);                                                                         \
    if (e_ != hipSuccess) {                                                                               \
      if (getenv("BAMBOO_DEBUG"))                                                                         \
        fprintf(stderr, "[bamboo] %s:%d HIP error %d: %s\n", __FILE__, __LINE__, (int)e_, hipGetErrorString(e_)); \
      (void)hipGetLastError();                                                                            \
      return BAMBOO_E_HIP;                                                                                \
    }                                                                                                     \
  } while (0)
}  // namespace

struct bamboo_ends {
  bamboo_cfg_t cfg;
  int V;
  EndsLayout l;
  const char* w[2];   // front, back parameters
  float* g[2];
  char* fstash;
  char* bstash;
  char* ws;
  std::vector<char> front_live;
  bool back_live;
};

extern "C" {

int ends_query_sizes(const bamboo_cfg_t* cfg, int32_t vocab, bamboo_ends_sizes_t* out) {
  const int v = check_cfg(cfg, vocab);
  if (v != BAMBOO_OK) return v;
  if (!out) return BAMBOO_E_ARG;
  const EndsLayout l = layout(*cfg, vocab);
  memset(out, 0, sizeof(*out));
  out->front_params = l.front_params;
  out->back_params = l.back_params;
  out->front_w = l.front_params * l.es;
  out->back_w = l.back_params * l.es;
  out->front_g = l.front_params * 4;
  out->back_g = l.back_params * 4;
  out->front_stash = l.fs_bytes * (uint64_t)cfg->M;
  out->back_stash = l.bs_bytes;
  out->workspace = l.ws_bytes;
  return BAMBOO_OK;
}

int ends_init(const bamboo_cfg_t* cfg, int32_t vocab, const bamboo_ends_sizes_t* sizes, const void* front_w,
              void* front_g, const void* back_w, void* back_g, void* front_stash, void* back_stash, void* workspace,
              bamboo_ends_t** out) {
  bamboo_ends_sizes_t need;
  const int v = ends_query_sizes(cfg, vocab, &need);
  if (v != BAMBOO_OK) return v;
  if (!sizes || !out || !front_w || !front_g || !back_w || !back_g || !front_stash || !back_stash || !workspace)
    return BAMBOO_E_ARG;
  if (sizes->front_w < need.front_w || sizes->back_w < need.back_w || sizes->front_g < need.front_g ||
      sizes->back_g < need.back_g || sizes->front_stash < need.front_stash || sizes->back_stash < need.back_stash ||
      sizes->workspace < need.workspace)
    return BAMBOO_E_ARG;
  const void* ptrs[] = {front_w, front_g, back_w, back_g, front_stash, back_stash, workspace};
  for (const void* p : ptrs)
    if (((uintptr_t)p) % kAlign) return BAMBOO_E_ARG;
  bamboo_ends* e = new (std::nothrow) bamboo_ends();
  if (!e) return BAMBOO_E_NOMEM;
  try {
    e->front_live.assign(cfg->M, 0);
  } catch (const std::bad_alloc&) {
    delete e;
    return BAMBOO_E_NOMEM;
  }
  e->cfg = *cfg;
  e->V = vocab;
  e->l = layout(*cfg, vocab);
  e->w[0] = (const char*)front_w;
  e->w[1] = (const char*)back_w;
  e->g[0] = (float*)front_g;
  e->g[1] = (float*)back_g;
  e->fstash = (char*)front_stash;
  e->bstash = (char*)back_stash;
  e->ws = (char*)workspace;
  e->back_live = false;
  *out = e;
  return BAMBOO_OK;
}

int ends_begin_iteration(bamboo_ends_t* e) {
  if (!e) return BAMBOO_E_ARG;
  std::fill(e->front_live.begin(), e->front_live.end(), 0);
  e->back_live = false;
  return BAMBOO_OK;
}

int ends_front_fwd(bamboo_ends_t* e, int32_t k, const int32_t* ids, void* x0, void* stream) {
  if (!e || !ids || !x0) return BAMBOO_E_ARG;
  if (k < 0 || k >= e->cfg.M) return BAMBOO_E_BADMB;
  const bamboo_cfg_t& c = e->cfg;
  const EndsLayout& l = e->l;
  const int T = c.micro_batch * c.seq, H = c.hidden;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();
  char* slot = e->fstash + (uint64_t)k * l.fs_bytes;
  int* ids_kept = (int*)(slot + l.fs_ids);
  ENDCHK(hipMemcpyAsync(ids_kept, ids, (uint64_t)T * 4, hipMemcpyDeviceToDevice, s));
  const void* Etok = e->w[0] + l.f_tok * l.es;
  const void* Epos = e->w[0] + l.f_pos * l.es;
  if (c.arch == BAMBOO_ARCH_POST_LN_ENCODER) {
    void* ev = slot + l.fs_e;
    ENDCHK(launch_embed_fwd(s, c.dtype, T, c.seq, H, e->V, ids_kept, Etok, Epos, ev));
    ENDCHK(launch_layernorm_fwd(s, c.dtype, T, H, c.ln_eps, ev, e->w[0] + l.f_g * l.es, e->w[0] + l.f_b * l.es, x0,
                                (float*)(slot + l.fs_stats)));
  } else {
    ENDCHK(launch_embed_fwd(s, c.dtype, T, c.seq, H, e->V, ids_kept, Etok, Epos, x0));
  }
  e->front_live[k] = 1;
  return BAMBOO_OK;
}

int ends_front_bwd(bamboo_ends_t* e, int32_t k, const void* dx0, void* stream) {
  if (!e || !dx0) return BAMBOO_E_ARG;
  if (k < 0 || k >= e->cfg.M || !e->front_live[k]) return BAMBOO_E_BADMB;
  const bamboo_cfg_t& c = e->cfg;
  const EndsLayout& l = e->l;
  const int T = c.micro_batch * c.seq, H = c.hidden;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();
  char* slot = e->fstash + (uint64_t)k * l.fs_bytes;
  const void* de = dx0;
  if (c.arch == BAMBOO_ARCH_POST_LN_ENCODER) {
    void* d = e->ws + l.ws_d;
    ENDCHK(launch_layernorm_bwd(s, c.dtype, T, H, dx0, slot + l.fs_e, (const float*)(slot + l.fs_stats),
                                e->w[0] + l.f_g * l.es, nullptr, d, e->g[0] + l.f_g, e->g[0] + l.f_b,
                                (float*)(e->ws + l.ws_partial)));
    de = d;
  }
  ENDCHK(launch_embed_bwd(s, c.dtype, T, c.seq, H, e->V, (const int*)(slot + l.fs_ids), de, e->g[0] + l.f_tok,
                          e->g[0] + l.f_pos));
  e->front_live[k] = 0;
  return BAMBOO_OK;
}

int ends_back_fwd(bamboo_ends_t* e, const void* y, const int32_t* labels, float* loss, void* stream) {
  if (!e || !y || !labels || !loss) return BAMBOO_E_ARG;
  const bamboo_cfg_t& c = e->cfg;
  const EndsLayout& l = e->l;
  const int T = c.micro_batch * c.seq, H = c.hidden, V = e->V;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();
  char* b = e->bstash;
  ENDCHK(hipMemcpyAsync(b + l.bs_y, y, (uint64_t)T * H * l.es, hipMemcpyDeviceToDevice, s));
  ENDCHK(hipMemcpyAsync(b + l.bs_labels, labels, (uint64_t)T * 4, hipMemcpyDeviceToDevice, s));
  const void* hf = b + l.bs_y;
  if (c.arch == BAMBOO_ARCH_PRE_LN_CAUSAL) {   // the decoder's final LayerNorm
    ENDCHK(launch_layernorm_fwd(s, c.dtype, T, H, c.ln_eps, b + l.bs_y, e->w[1] + l.b_g * l.es, e->w[1] + l.b_b * l.es,
                                b + l.bs_hf, (float*)(b + l.bs_stats)));
    hf = b + l.bs_hf;
  }
  GemmDesc d;
  memset(&d, 0, sizeof(d));
  d.A = hf; d.B = e->w[1] + l.b_head * l.es; d.C = b + l.bs_logits; d.M = T; d.N = V; d.K = H;
  d.a_sm = H; d.a_sk = 1; d.b_sk = V; d.b_sn = 1; d.epi = EPI_STORE;
  ENDCHK(launch_gemm(s, c.dtype, d));
  ENDCHK(launch_xent_fwd(s, c.dtype, T, V, b + l.bs_logits, (const int*)(b + l.bs_labels), (float*)(b + l.bs_lse),
                         (float*)(b + l.bs_tok)));
  ENDCHK(launch_ordered_sum(s, T, (const float*)(b + l.bs_tok), 1.0f / (float)T, loss));
  e->back_live = true;
  return BAMBOO_OK;
}

int ends_back_bwd(bamboo_ends_t* e, void* gy, void* stream) {
  if (!e || !gy) return BAMBOO_E_ARG;
  if (!e->back_live) return BAMBOO_E_STATE;
  const bamboo_cfg_t& c = e->cfg;
  const EndsLayout& l = e->l;
  const int T = c.micro_batch * c.seq, H = c.hidden, V = e->V;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();
  char* b = e->bstash;
  const bool dec = c.arch == BAMBOO_ARCH_PRE_LN_CAUSAL;
  const void* hf = dec ? b + l.bs_hf : b + l.bs_y;
  void* dl = b + l.bs_logits;   // the logits become their gradient
  ENDCHK(launch_xent_bwd(s, c.dtype, T, V, dl, (const int*)(b + l.bs_labels), (const float*)(b + l.bs_lse),
                         1.0f / (float)T, dl));
  GemmDesc d;
  // dW_head[H,V] += hf^T dlogits
  memset(&d, 0, sizeof(d));
  d.A = hf; d.B = dl; d.C = e->g[1] + l.b_head; d.M = H; d.N = V; d.K = T;
  d.a_sm = 1; d.a_sk = H; d.b_sk = V; d.b_sn = 1; d.epi = EPI_ACC_F32;
  ENDCHK(launch_gemm(s, c.dtype, d));
  // dhf[T,H] = dlogits W_head^T
  void* dhf = dec ? (void*)(e->ws + l.ws_d) : gy;
  memset(&d, 0, sizeof(d));
  d.A = dl; d.B = e->w[1] + l.b_head * l.es; d.C = dhf; d.M = T; d.N = H; d.K = V;
  d.a_sm = V; d.a_sk = 1; d.b_sk = 1; d.b_sn = V; d.epi = EPI_STORE;
  ENDCHK(launch_gemm(s, c.dtype, d));
  if (dec)
    ENDCHK(launch_layernorm_bwd(s, c.dtype, T, H, dhf, b + l.bs_y, (const float*)(b + l.bs_stats),
                                e->w[1] + l.b_g * l.es, nullptr, gy, e->g[1] + l.b_g, e->g[1] + l.b_b,
                                (float*)(e->ws + l.ws_partial)));
  e->back_live = false;
  return BAMBOO_OK;
}

int ends_destroy(bamboo_ends_t* e) {
  if (!e) return BAMBOO_E_ARG;
  delete e;
  return BAMBOO_OK;
}

}  // extern "C"
