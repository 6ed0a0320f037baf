/*
 * bamboo_debug.h -- measurement, tuning and inspection hooks of the Bamboo stage library.
 *
 * Nothing here is part of the method (arXiv 2204.12013, Section 5): these calls exist so that the
 * kernels can be timed one by one, their launch shapes forced in tests, and intermediate results of a
 * backward pass read back for parity checks.  A training loop needs bamboo_stage.h only.
 * Conventions as in bamboo_stage.h (plain C types, device pointers owned by the caller, negative
 * bamboo_status on error).
 */
#ifndef BAMBOO_DEBUG_H
#define BAMBOO_DEBUG_H

#include <stdint.h>

#include "bamboo_stage.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-launch-site timing for roofline measurements.  stage_profile(st, 1) clears earlier records and
 * brackets every later kernel launch with a HIP event pair on the launch's own stream;
 * stage_profile(st, 0) stops.  stage_profile_read synchronises, then reports for one site the summed
 * launch durations in ms, the number of launches and the summed algorithmic work (flops for GEMM and
 * attention sites, bytes for the others).  The GEMM sites are the call sites of one layer pass, so
 * that a report can name the single launch that dominates. */
enum bamboo_kernel_class {
  BAMBOO_K_GEMM_QKV = 0,        /* qkv = ain Wqkv + bqkv */
  BAMBOO_K_GEMM_ATTN_OUT = 1,   /* r1 = x + ctx Wo + bo */
  BAMBOO_K_GEMM_FFN1 = 2,       /* GELU(fin W1 + b1) and its derivative */
  BAMBOO_K_GEMM_FFN2 = 3,       /* fin|r1 + g W2 + b2 */
  BAMBOO_K_DGRAD_FFN2 = 4,      /* dh = (df W2^T) * GELU'(h), with the column sums of dh */
  BAMBOO_K_DGRAD_FFN1 = 5,      /* dh W1^T (+ residual) */
  BAMBOO_K_DGRAD_ATTN_OUT = 6,  /* dctx = da Wo^T */
  BAMBOO_K_DGRAD_QKV = 7,       /* dqkv Wqkv^T (+ residual) */
  BAMBOO_K_WGRAD_GROUP = 8,     /* the four weight gradients of a layer (one launch where grouped) */
  BAMBOO_K_ATTN_FWD = 9,
  BAMBOO_K_ATTN_BWD = 10,
  BAMBOO_K_LN_FWD = 11,
  BAMBOO_K_LN_BWD = 12,
  BAMBOO_K_COLSUM = 13,
  BAMBOO_K_COUNT = 14
};
int stage_profile(bamboo_stage_t* st, int enable);
int stage_profile_read(bamboo_stage_t* st, int32_t kernel_class, double* total_ms, int64_t* launches, double* work);

/* Byte offsets, inside the workspace passed to stage_init, of the lane-0 buffers a backward pass
 * leaves its intermediate gradients in (storage dtype, row-major), so that a test can read them
 * after stage_bwd / shadow_bwd_brc of a one-layer stack has finished:
 * out[0] dh    [T,F]  gradient at the FFN pre-activation
 * out[1] d1    [T,H]  scratch of the input-gradient GEMMs (pre-LN: last holds dqkv Wqkv^T)
 * out[2] d2    [T,H]  pre-LN: gradient at the attention block's output; post-LN: input of LN1's backward
 * out[3] d3    [T,H]  post-LN: gradient at the FFN output
 * out[4] dctx  [T,H]  gradient at the attention context
 * out[5] dqkv  [T,3H] gradient at the projected queries | keys | values
 * out[6] bytes of the lane-0 area.  host pointers. */
int stage_workspace_fields(const bamboo_cfg_t* cfg, uint64_t out[7]);

/* Plain device copy of `bytes` bytes (multiple of 16, 16-byte aligned pointers) by a kernel with a
 * name of its own.  Its known traffic calibrates the HBM byte counters read for the other kernels. */
int bk_copy(const void* src, void* dst, uint64_t bytes, void* stream);

/* Choose the output tile of the MFMA GEMM kernel for all later calls in this process.
 * code = 10*WM + WN selects a (64*WM) x (64*WN) tile, one of 44, 43, 42, 24, 22, 11; 0 restores the
 * automatic choice.  Returns the previous code, or BAMBOO_E_ARG for a code that is not offered.
 * Process-wide: the caller must not change it while another thread launches. */
int bk_gemm_tile(int code);

/* Force the depth of the LDS slice ring of the pipelined MFMA GEMM kernel (2, 3 or 4 buffers; a
 * depth that does not fit the tile's LDS budget or exceeds the number of K slices falls back to the
 * next smaller one); 0 restores the automatic choice.  Returns the previous value, or BAMBOO_E_ARG.
 * Process-wide, like bk_gemm_tile. */
int bk_gemm_stages(int n);

#ifdef __cplusplus
}
#endif
#endif /* BAMBOO_DEBUG_H */
