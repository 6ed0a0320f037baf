/*
 * bamboo_ends.h -- C ABI of the two ends of the model, for the wrap-around stage
 * (arXiv 2204.12013, Section 5.1: the first node's layers are replicated on the
 * last node, which "fetches input samples directly" to run redundant computation
 * for it).  The last stage therefore works on what no middle stage sees: token
 * ids, through the first stage's embedding (front), and labels, through the LM
 * head and the loss that its own backward starts from (back).  The paper leaves
 * both to the models it trains (Section 7, Table 1); they are the textbook ones:
 *
 *   front   e[t] = E_tok[ids[t]] + E_pos[t mod seq]
 *           post-LN encoder: x0 = LayerNorm(e; g_e, b_e)     pre-LN decoder: x0 = e
 *   back    post-LN encoder: hf = y        pre-LN decoder: hf = LayerNorm(y; g_f, b_f)
 *           logits = hf W_head, W_head [H, V]
 *           loss = mean over the micro-batch's tokens of log sum_v exp(logits[t,v]) - logits[t, labels[t]]
 *
 * An ends object goes with one bamboo_stage_t configured with cfg.wrap = 1; the caller
 * composes them per instruction, on the stream the stage uses for it:
 *   FWD(k) = stage_fwd(k, x, y);            ends_back_fwd(y, labels_k, loss_k)          main stream
 *   BWD(k) = ends_back_bwd(gy);             stage_bwd(k, gy, gx)                        main stream
 *   FRC(k) = ends_front_fwd(k, ids_k, x0);  shadow_fwd_frc(k, x0, z)     FRC stream (main after failover_merge)
 *   BRC(k) = shadow_bwd_brc(k, g1_k, dx0);  ends_front_bwd(k, dx0)                      main stream
 *
 * Conventions as in bamboo_stage.h: device pointers owned by the caller, 256-byte
 * aligned; streams as void*; calls enqueue and return; 0 or a negative bamboo_status.
 * Parameters are flat, in the storage dtype; gradients fp32 with the same layout:
 *   front: E_tok [V,H] | E_pos [seq,H] | g_e [H] | b_e [H]     (the last two only for the post-LN encoder)
 *   back:  g_f [H] | b_f [H] | W_head [H,V]                    (the first two only for the pre-LN decoder)
 * ids and labels are int32 [tokens]; values outside [0, V) are clamped into the range.
 */
#ifndef BAMBOO_ENDS_H
#define BAMBOO_ENDS_H

#include <stdint.h>

#include "bamboo_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bamboo_ends bamboo_ends_t; /* opaque, host side */

typedef struct {
  uint64_t front_params, back_params; /* elements */
  uint64_t front_w, back_w;           /* bytes, storage dtype */
  uint64_t front_g, back_g;           /* bytes, fp32 */
  uint64_t front_stash;               /* M slots: the ids and, for the encoder, e and the LayerNorm statistics */
  uint64_t back_stash;                /* one slot (the last stage has one micro-batch in flight): the stage
                                         output, the LayerNorm statistics and output, the logits [tokens, V]
                                         (overwritten by their gradient in the backward), lse, per-token loss,
                                         the labels */
  uint64_t workspace;                 /* scratch of the two backwards */
} bamboo_ends_sizes_t;

/* vocab: V, a multiple of 8.  BAMBOO_E_BADCFG for a bad cfg or vocab. */
int ends_query_sizes(const bamboo_cfg_t* cfg, int32_t vocab, bamboo_ends_sizes_t* out);

/* Creates the host-side object; keeps the pointers.  sizes: what the caller allocated (each >= the
 * queried size).  Allocates no device memory. */
int ends_init(const bamboo_cfg_t* cfg, int32_t vocab, const bamboo_ends_sizes_t* sizes, const void* front_w,
              void* front_g, const void* back_w, void* back_g, void* front_stash, void* back_stash, void* workspace,
              bamboo_ends_t** out);

/* x0 [tokens,H] = front(ids) for micro-batch k (slot k of the front stash keeps what the backward needs). */
int ends_front_fwd(bamboo_ends_t* e, int32_t k, const int32_t* ids, void* x0, void* stream);
/* front_g += gradients from dx0 [tokens,H], the gradient at the front's output, for micro-batch k.
 * BAMBOO_E_BADMB if ends_front_fwd(k) has not run since the last ends_begin_iteration. */
int ends_front_bwd(bamboo_ends_t* e, int32_t k, const void* dx0, void* stream);
/* loss[0] (device fp32) = mean token loss of the micro-batch whose stage output is y [tokens,H]. */
int ends_back_fwd(bamboo_ends_t* e, const void* y, const int32_t* labels, float* loss, void* stream);
/* gy [tokens,H] = gradient of that loss at y; back_g += the head's gradients.  BAMBOO_E_STATE without a
 * forward before it. */
int ends_back_bwd(bamboo_ends_t* e, void* gy, void* stream);
/* forgets which slots hold a forward (does not touch gradients) */
int ends_begin_iteration(bamboo_ends_t* e);
int ends_destroy(bamboo_ends_t* e);

#ifdef __cplusplus
}
#endif
#endif
