/*
 * bamboo_kernels.h -- C ABI of the individual layer kernels the Bamboo stage
 * is built from (arXiv 2204.12013, Section 5.1: FNC/BNC and FRC/BRC are the
 * same layer computation; the paper leaves the layer math to the models it
 * trains, Section 7 Table 1: BERT-Large, GPT-2).  Exposed so that each kernel
 * can be checked and timed on its own.
 *
 * All data pointers are device pointers owned by the caller; `stream` is a
 * hipStream_t passed as void*.  Calls enqueue and return.  dtype: 0 fp32,
 * 1 bf16 storage with fp32 accumulation.  impl: 0 automatic (MFMA kernel when it
 * covers the shape, vector-ALU kernel otherwise), 1 vector-ALU kernel,
 * 2 MFMA kernel (BAMBOO_E_STATE if it does not cover the shape).
 * Return: 0 or a negative bamboo_status (see bamboo_stage.h).
 * Tensors are row-major; "tokens" T = batch * seq.
 */
#ifndef BAMBOO_KERNELS_H
#define BAMBOO_KERNELS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Y[T,N] = X[T,K] W[K,N] + bias[N] (+ res[T,N] if res != NULL).
 * If gelu_out != NULL (and res == NULL), with h = X W + bias kept in fp32:
 * gelu_out[T,N] = GELU(h) (erf form) and Y[T,N] = GELU'(h), the factor the
 * backward multiplies the incoming gradient by (so GELU is evaluated once, in
 * the forward, and the pre-activation itself is not kept). */
int bk_linear_fwd(int dtype, int impl, int T, int N, int K, const void* X, const void* W, const void* bias,
                  const void* res, void* Y, void* gelu_out, void* stream);

/* dX[T,K] = dY[T,N] W[K,N]^T (+ res[T,K] if res != NULL).
 * If mul != NULL (and res == NULL): dX = (dY W^T) * mul[T,K] elementwise (the
 * backward through an activation whose derivative the forward stored). */
int bk_linear_bwd_input(int dtype, int impl, int T, int K, int N, const void* dY, const void* W, const void* res,
                        const void* mul, void* dX, void* stream);

/* dW[K,N] (fp32) += X[T,K]^T dY[T,N]; if db != NULL also db[N] (fp32) += sum over
 * tokens of dY (the bias gradient of the same linear layer), with
 * partial = fp32 scratch of bk_colsum_scratch_floats(N) floats. */
int bk_linear_bwd_weight(int dtype, int impl, int T, int K, int N, const void* X, const void* dY, float* dW,
                         float* db, float* partial, void* stream);

/* n (1..4) independent weight gradients in one go: dW[i][K[i],N[i]] (fp32) += X[i][T[i],K[i]]^T dY[i][T[i],N[i]].
 * T, K, N: host int arrays; X, dY, dW: host arrays of device pointers.  Where the MFMA kernel covers all
 * of them with one tile shape (bf16, T a multiple of 64 and >= 192, K and N multiples of 8) they run as
 * ONE launch whose workgroups are dealt over the problems, so that problems that do not fill the chip on
 * their own share its rounds; otherwise one launch each.  The results do not depend on which. */
int bk_linear_bwd_weight_group(int dtype, int n, const int* T, const int* K, const int* N, const void* const* X,
                               const void* const* dY, float* const* dW, void* stream);

/* out[N] (fp32) += sum over tokens of A[T,N]; partial: fp32 scratch of
 * bk_colsum_scratch_floats(N) floats.  Fixed summation order. */
int bk_colsum_acc(int dtype, int T, int N, const void* A, float* out, float* partial, void* stream);
uint64_t bk_colsum_scratch_floats(int N);

/* bk_colsum_acc for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same result as bk_colsum_acc (the same two kernels
 * in the same order), but the partial rows live in a device array inside the library (2 MiB per GPU,
 * held until the process ends) instead of a caller buffer; the call allocates and frees nothing.
 * A, out: device pointers as for bk_colsum_acc (out is added to).  BAMBOO_E_ARG if the shape needs
 * more than bk_colsum_static_max_floats() = 2^19 floats of partial rows (partial rows x N; the launch
 * shape keeps that product below 2^18 until a single row exceeds the array, i.e. every N <= 524288
 * fits with any T), decided before anything is launched.  All calls on one GPU share that GPU's array: calls that overlap on one GPU (two
 * streams, two threads) race; calls on one stream, one after the other, are safe, and nothing needs
 * clearing between them. */
int bk_colsum_acc_static(int dtype, int T, int N, const void* A, float* out, void* stream);
uint64_t bk_colsum_static_max_floats(void);

/* Softmax attention.  qkv[T,3H] = queries | keys | values, head h = columns
 * h*d..(h+1)*d-1 of each third; scores scaled by 1/sqrt(d); causal != 0 masks
 * keys after the query.  ctx[T,H]; lse[batch,heads,seq] fp32 = log-sum-exp of
 * the scaled scores of each row. */
int bk_attention_fwd(int dtype, int impl, int batch, int seq, int heads, int d, int causal, const void* qkv, void* ctx,
                     float* lse, void* stream);
/* dqkv[T,3H] from dctx[T,H], recomputing the probabilities from lse.
 * delta: fp32 scratch [batch,heads,seq]. */
int bk_attention_bwd(int dtype, int impl, int batch, int seq, int heads, int d, int causal, const void* qkv,
                     const void* ctx, const float* lse, const void* dctx, void* dqkv, float* delta, void* stream);

/* y = gamma * (r - mean) * rstd + beta per token row; stats[2t] = mean,
 * stats[2t+1] = rstd = 1/sqrt(biased variance + eps). */
int bk_layernorm_fwd(int dtype, int T, int H, float eps, const void* r, const void* gamma, const void* beta, void* y,
                     float* stats, void* stream);
/* dr = LayerNorm backward of dout (+ add[T,H] if add != NULL); dgamma, dbeta
 * (fp32) += their token sums.  partial: fp32 scratch of
 * bk_layernorm_bwd_scratch_floats(H) floats. */
int bk_layernorm_bwd(int dtype, int T, int H, const void* dout, const void* r, const float* stats, const void* gamma,
                     const void* add, void* dr, float* dgamma, float* dbeta, float* partial, void* stream);
uint64_t bk_layernorm_bwd_scratch_floats(int H);

/* One Adam step (Section 7 names the optimizer) over n parameters, n a multiple of 4, step >= 1:
 * g fp32 gradient; master, m, v fp32 master weights and moments, updated in place; w[n] (storage
 * dtype) = the new master weights rounded to storage.  All device pointers, 16-byte aligned. */
int bk_adam(int dtype, int64_t n, const float* g, float* master, float* m, float* v, void* w, float lr, float beta1,
            float beta2, float eps, int step, void* stream);

/* ---- the two ends of the model, worked on by the wrap-around stage only (Section 5.1: the last
 * node keeps the replica of the first node's layers and fetches the input samples itself).  The
 * paper does not spell them out; they are the textbook ends of the models it trains.
 *
 * Front: out[t,:] = E_tok[ids[t],:] + E_pos[t mod seq,:], the sum taken in fp32 and rounded to the
 * storage type.  ids: device int32 [T]; values outside [0, V) are clamped into the range (never
 * read out of bounds).  H a multiple of 8; E_tok [V,H], E_pos [seq,H], out [T,H] 32-byte aligned. */
int bk_embedding_fwd(int dtype, int T, int seq, int H, int V, const int32_t* ids, const void* E_tok, const void* E_pos,
                     void* out, void* stream);
/* dE_tok[V,H] (fp32) += rows of g[T,H] scattered by ids, dE_pos[seq,H] (fp32) += rows of g summed over
 * the samples.  No atomics: rows hit by several tokens are added in token order. */
int bk_embedding_bwd(int dtype, int T, int seq, int H, int V, const int32_t* ids, const void* g, float* dE_tok,
                     float* dE_pos, void* stream);
/* Back: per token t, lse[t] = log sum_v exp(logits[t,v]) and loss_tok[t] = lse[t] - logits[t,labels[t]]
 * (fp32, from the stored logits); V a multiple of 8, logits [T,V] 32-byte aligned. */
int bk_softmax_xent_fwd(int dtype, int T, int V, const void* logits, const int32_t* labels, float* lse,
                        float* loss_tok, void* stream);
/* dlogits[t,v] = (exp(logits[t,v] - lse[t]) - [v == labels[t]]) * scale; dlogits may be logits. */
int bk_softmax_xent_bwd(int dtype, int T, int V, const void* logits, const int32_t* labels, const float* lse,
                        float scale, void* dlogits, void* stream);
/* out[0] = scale * (in[0] + ... + in[n-1]) in a fixed order (the mean loss of a micro-batch). */
int bk_ordered_sum(int64_t n, const float* in, float scale, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BAMBOO_KERNELS_H */
