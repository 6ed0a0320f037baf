// C ABI of the individual kernels: argument checks and marshalling only.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/bamboo_debug.h"
#include "../../include/bamboo_kernels.h"
#include "../../include/bamboo_stage.h"
#include "common.h"

using namespace bamboo;

namespace {
int finish(hipError_t e) {
  if (e == hipSuccess) return BAMBOO_OK;
  if (getenv("BAMBOO_DEBUG")) fprintf(stderr, "[bamboo] HIP error %d: %s\n", (int)e, hipGetErrorString(e));
  (void)hipGetLastError();
  return e == hipErrorNotSupported ? BAMBOO_E_STATE : BAMBOO_E_HIP;
}
int run_gemm(int dtype, int impl, const GemmDesc& d, void* stream) {
  (void)hipGetLastError();  // an earlier, unrelated failure in this thread must not be blamed on this launch
  if (dtype != 0 && dtype != 1) return BAMBOO_E_ARG;
  if (d.M <= 0 || d.N <= 0 || d.K <= 0 || !d.A || !d.B || !d.C) return BAMBOO_E_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (impl == 1) return finish(launch_gemm_simple(s, dtype, d));
  if (impl == 2) return dtype == 1 ? finish(launch_gemm_mfma(s, d)) : BAMBOO_E_STATE;
  if (impl != 0) return BAMBOO_E_ARG;
  return finish(launch_gemm(s, dtype, d));
}
}  // namespace

extern "C" {

int bk_linear_fwd(int dtype, int impl, int T, int N, int K, const void* X, const void* W, const void* bias,
                  const void* res, void* Y, void* gelu_out, void* stream) {
  if (!bias || (res && gelu_out)) return BAMBOO_E_ARG;   // with gelu_out: Y = GELU'(h), gelu_out = GELU(h)
  GemmDesc d;
  memset(&d, 0, sizeof(d));
  d.A = X; d.B = W; d.C = Y; d.M = T; d.N = N; d.K = K;
  d.a_sm = K; d.a_sk = 1; d.b_sk = N; d.b_sn = 1;
  d.bias = bias; d.res = res; d.aux_out = gelu_out;
  d.epi = gelu_out ? EPI_BIAS_GELU : (res ? EPI_BIAS_RES : EPI_BIAS);
  return run_gemm(dtype, impl, d, stream);
}

int bk_linear_bwd_input(int dtype, int impl, int T, int K, int N, const void* dY, const void* W, const void* res,
                        const void* mul, void* dX, void* stream) {
  if (mul && res) return BAMBOO_E_ARG;
  GemmDesc d;
  memset(&d, 0, sizeof(d));
  d.A = dY; d.B = W; d.C = dX; d.M = T; d.N = K; d.K = N;
  d.a_sm = N; d.a_sk = 1; d.b_sk = 1; d.b_sn = N;
  d.res = res; d.aux_in = mul;
  d.epi = mul ? EPI_MUL : (res ? EPI_RES : EPI_STORE);
  return run_gemm(dtype, impl, d, stream);
}

int bk_linear_bwd_weight(int dtype, int impl, int T, int K, int N, const void* X, const void* dY, float* dW,
                         float* db, float* partial, void* stream) {
  if (db != nullptr && partial == nullptr) return BAMBOO_E_ARG;
  GemmDesc d;
  memset(&d, 0, sizeof(d));
  d.A = X; d.B = dY; d.C = dW; d.M = K; d.N = N; d.K = T;
  d.a_sm = 1; d.a_sk = K; d.b_sk = N; d.b_sn = 1;
  d.epi = EPI_ACC_F32;
  d.colsum_out = db; d.colsum_partial = partial;
  if (impl != 0 && db != nullptr) {   // a forced kernel bypasses launch_gemm: the column sum is launched here
    (void)hipGetLastError();
    const int rc = finish(launch_colsum_acc((hipStream_t)stream, dtype, T, N, dY, db, partial));
    if (rc != BAMBOO_OK) return rc;
    d.colsum_out = nullptr;
  }
  return run_gemm(dtype, impl, d, stream);
}

int bk_linear_bwd_weight_group(int dtype, int n, const int* T, const int* K, const int* N, const void* const* X,
                               const void* const* dY, float* const* dW, void* stream) {
  if ((dtype != 0 && dtype != 1) || n < 1 || n > GemmGroup::MAX || !T || !K || !N || !X || !dY || !dW) return BAMBOO_E_ARG;
  GemmDesc d[GemmGroup::MAX];
  memset(d, 0, sizeof(d));
  for (int i = 0; i < n; ++i) {
    if (T[i] <= 0 || K[i] <= 0 || N[i] <= 0 || !X[i] || !dY[i] || !dW[i]) return BAMBOO_E_ARG;
    d[i].A = X[i]; d[i].B = dY[i]; d[i].C = dW[i]; d[i].M = K[i]; d[i].N = N[i]; d[i].K = T[i];
    d[i].a_sm = 1; d[i].a_sk = K[i]; d[i].b_sk = N[i]; d[i].b_sn = 1; d[i].epi = EPI_ACC_F32;
  }
  (void)hipGetLastError();
  return finish(launch_gemm_group((hipStream_t)stream, dtype, d, n));
}

int bk_colsum_acc(int dtype, int T, int N, const void* A, float* out, float* partial, void* stream) {
  if ((dtype != 0 && dtype != 1) || T <= 0 || N <= 0 || N % 2 || !A || !out || !partial) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_colsum_acc((hipStream_t)stream, dtype, T, N, A, out, partial));
}
uint64_t bk_colsum_scratch_floats(int N) { return colsum_partial_floats(N); }

static int attn_desc(AttnDesc& a, int dtype, int batch, int seq, int heads, int d, int causal) {
  if ((dtype != 0 && dtype != 1) || batch <= 0 || seq <= 0 || heads <= 0 || d <= 0 || d > 128) return BAMBOO_E_ARG;
  memset(&a, 0, sizeof(a));
  a.B = batch; a.S = seq; a.heads = heads; a.d = d; a.causal = causal != 0;
  return BAMBOO_OK;
}

int bk_attention_fwd(int dtype, int impl, int batch, int seq, int heads, int d, int causal, const void* qkv, void* ctx,
                     float* lse, void* stream) {
  AttnDesc a;
  if (attn_desc(a, dtype, batch, seq, heads, d, causal) != BAMBOO_OK || !qkv || !ctx || !lse) return BAMBOO_E_ARG;
  a.qkv = qkv; a.ctx = ctx; a.lse = lse;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();
  if (impl == 1) return finish(launch_attention_fwd_simple(s, dtype, a));
  if (impl == 2) return dtype == 1 ? finish(launch_attention_fwd_mfma(s, a)) : BAMBOO_E_STATE;
  if (impl != 0) return BAMBOO_E_ARG;
  return finish(launch_attention_fwd(s, dtype, a));
}

int bk_attention_bwd(int dtype, int impl, int batch, int seq, int heads, int d, int causal, const void* qkv,
                     const void* ctx, const float* lse, const void* dctx, void* dqkv, float* delta, void* stream) {
  AttnDesc a;
  if (attn_desc(a, dtype, batch, seq, heads, d, causal) != BAMBOO_OK || !qkv || !ctx || !lse || !dctx || !dqkv ||
      !delta)
    return BAMBOO_E_ARG;
  a.qkv = qkv; a.ctx = (void*)ctx; a.lse = (float*)lse; a.dctx = dctx; a.dqkv = dqkv; a.delta = delta;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();
  if (impl == 1) return finish(launch_attention_bwd_simple(s, dtype, a));
  if (impl == 2) return dtype == 1 ? finish(launch_attention_bwd_mfma(s, a)) : BAMBOO_E_STATE;
  if (impl != 0) return BAMBOO_E_ARG;
  return finish(launch_attention_bwd(s, dtype, a));
}

int bk_layernorm_fwd(int dtype, int T, int H, float eps, const void* r, const void* gamma, const void* beta, void* y,
                     float* stats, void* stream) {
  if ((dtype != 0 && dtype != 1) || T <= 0 || H <= 0 || H % 8 || !r || !gamma || !beta || !y || !stats)
    return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_layernorm_fwd((hipStream_t)stream, dtype, T, H, eps, r, gamma, beta, y, stats));
}

int bk_layernorm_bwd(int dtype, int T, int H, const void* dout, const void* r, const float* stats, const void* gamma,
                     const void* add, void* dr, float* dgamma, float* dbeta, float* partial, void* stream) {
  if ((dtype != 0 && dtype != 1) || T <= 0 || H <= 0 || H % 8 || !dout || !r || !stats || !gamma || !dr || !dgamma ||
      !dbeta || !partial)
    return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_layernorm_bwd((hipStream_t)stream, dtype, T, H, dout, r, stats, gamma, add, dr, dgamma, dbeta,
                                     partial));
}
uint64_t bk_layernorm_bwd_scratch_floats(int H) { return ln_bwd_partial_floats(H); }

int bk_copy(const void* src, void* dst, uint64_t bytes, void* stream) {
  if (!src || !dst || bytes % 16 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_calibration_copy((hipStream_t)stream, src, dst, (size_t)bytes));
}

int bk_adam(int dtype, int64_t n, const float* g, float* master, float* m, float* v, void* w, float lr, float beta1,
            float beta2, float eps, int step, void* stream) {
  if (dtype != 0 && dtype != 1) return BAMBOO_E_ARG;
  if (n <= 0 || n % 4 || step < 1 || !g || !master || !m || !v || !w) return BAMBOO_E_ARG;
  const void* ptrs[] = {g, master, m, v, w};
  for (const void* p : ptrs)
    if (((uintptr_t)p) & 15) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_adam((hipStream_t)stream, dtype, (long)n, g, master, m, v, w, lr, beta1, beta2, eps, step));
}

int bk_embedding_fwd(int dtype, int T, int seq, int H, int V, const int32_t* ids, const void* E_tok, const void* E_pos,
                     void* out, void* stream) {
  if ((dtype != 0 && dtype != 1) || T <= 0 || seq <= 0 || H <= 0 || H % 8 || V <= 0) return BAMBOO_E_ARG;
  if (!ids || !E_tok || !E_pos || !out) return BAMBOO_E_ARG;
  if (((uintptr_t)E_tok | (uintptr_t)E_pos | (uintptr_t)out) & 31) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_embed_fwd((hipStream_t)stream, dtype, T, seq, H, V, ids, E_tok, E_pos, out));
}

int bk_embedding_bwd(int dtype, int T, int seq, int H, int V, const int32_t* ids, const void* g, float* dE_tok,
                     float* dE_pos, void* stream) {
  if ((dtype != 0 && dtype != 1) || T <= 0 || seq <= 0 || T % seq || H <= 0 || V <= 0) return BAMBOO_E_ARG;
  if (!ids || !g || !dE_tok || !dE_pos) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_embed_bwd((hipStream_t)stream, dtype, T, seq, H, V, ids, g, dE_tok, dE_pos));
}

int bk_softmax_xent_fwd(int dtype, int T, int V, const void* logits, const int32_t* labels, float* lse,
                        float* loss_tok, void* stream) {
  if ((dtype != 0 && dtype != 1) || T <= 0 || V <= 0 || V % 8) return BAMBOO_E_ARG;
  if (!logits || !labels || !lse || !loss_tok || ((uintptr_t)logits & 31)) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_xent_fwd((hipStream_t)stream, dtype, T, V, logits, labels, lse, loss_tok));
}

int bk_softmax_xent_bwd(int dtype, int T, int V, const void* logits, const int32_t* labels, const float* lse,
                        float scale, void* dlogits, void* stream) {
  if ((dtype != 0 && dtype != 1) || T <= 0 || V <= 0 || V % 8) return BAMBOO_E_ARG;
  if (!logits || !labels || !lse || !dlogits || (((uintptr_t)logits | (uintptr_t)dlogits) & 31)) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_xent_bwd((hipStream_t)stream, dtype, T, V, logits, labels, lse, scale, dlogits));
}

int bk_ordered_sum(int64_t n, const float* in, float scale, float* out, void* stream) {
  if (n <= 0 || !in || !out) return BAMBOO_E_ARG;
  (void)hipGetLastError();
  return finish(launch_ordered_sum((hipStream_t)stream, (long)n, in, scale, out));
}

int bk_gemm_tile(int code) {
  if (!gemm_tile_code_valid(code)) return BAMBOO_E_ARG;
  return set_gemm_tile(code);
}

int bk_gemm_stages(int n) {
  if (n != 0 && (n < 2 || n > 4)) return BAMBOO_E_ARG;
  return set_gemm_stages(n);
}

}  // extern "C"
