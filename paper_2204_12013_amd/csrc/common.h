// Shared device helpers and the internal launcher interface of the Bamboo
// stage library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

typedef __bf16 bf16_t;

namespace bamboo {

// ---- storage <-> fp32 ------------------------------------------------------
template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }  // RNE

// value after a round trip through the storage type
template <typename T> __device__ __forceinline__ float round_storage(float v) { return to_f32<T>(from_f32<T>(v)); }

// erf-form GELU and its derivative (fp32)
__device__ __forceinline__ float gelu_f(float h) { return 0.5f * h * (1.0f + erff(h * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float h) {
  return 0.5f * (1.0f + erff(h * 0.70710678118654752f)) + h * __expf(-0.5f * h * h) * 0.39894228040143268f;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- per-process launch state ------------------------------------------------
// Set up once per device by whichever thread gets there first (stages driven from different threads
// share it).
constexpr int kMaxDevices = 64;
inline int current_device_index() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  return dev < 0 || dev >= kMaxDevices ? 0 : dev;
}
// A kernel that uses more than 64 KB of dynamic LDS has to be told so once per device.
template <auto KERNEL, int BYTES>
inline hipError_t ensure_lds_attribute() {
  static std::once_flag once[kMaxDevices];
  static hipError_t result[kMaxDevices];
  const int dev = current_device_index();
  std::call_once(once[dev], [dev]() {
    result[dev] = hipFuncSetAttribute((const void*)KERNEL, hipFuncAttributeMaxDynamicSharedMemorySize, BYTES);
  });
  return result[dev];
}

// ---- GEMM ------------------------------------------------------------------
// C[M,N] = op(A)[M,K] * op(B)[K,N] with an epilogue; fp32 accumulation.
// A(m,k) sits at A[m*a_sm + k*a_sk], B(k,n) at B[k*b_sk + n*b_sn]; exactly one
// stride of each operand is 1.  C, res, aux are row-major with leading
// dimension N.
enum Epilogue : int {
  EPI_STORE = 0,      // C = acc
  EPI_BIAS = 1,       // C = acc + bias[n]
  EPI_BIAS_RES = 2,   // C = acc + bias[n] + res[m,n]
  EPI_BIAS_GELU = 3,  // h = acc + bias[n] (fp32): aux_out = gelu(h), C = gelu'(h)
  EPI_RES = 4,        // C = acc + res[m,n]
  EPI_MUL = 5,        // C = acc * aux_in[m,n]
  EPI_ACC_F32 = 6     // C (fp32) += acc
};

struct GemmDesc {
  const void* A;
  const void* B;
  void* C;
  int M, N, K;
  long a_sm, a_sk, b_sk, b_sn;
  int epi;
  const void* bias;     // [N] storage dtype
  const void* res;      // [M,N]
  const void* aux_in;   // [M,N]
  void* aux_out;        // [M,N]
  // weight-gradient form only (honoured by launch_gemm, not by the kernels):
  // colsum_out[n] (fp32) += sum_k B(k,n), i.e. the bias gradient that belongs to
  // the same dY; colsum_partial is scratch of colsum_partial_floats(N) floats
  float* colsum_out;
  float* colsum_partial;
  // EPI_MUL only: tile_colsum (device fp32, reduce_max_partials() rows of N) receives one row of column
  // sums of the stored outputs per row of output tiles, and *tile_colsum_parts (host) the number of rows
  // written -- the bias gradient of the linear layer whose pre-activation gradient this GEMM produces,
  // without reading the output again.  Honoured by launch_gemm (kernels that cannot do it get a
  // column-sum launch behind them).
  float* tile_colsum;
  int* tile_colsum_parts;
  // Launch hint (does not change the result): the launch shares the chip with another stream's kernels, which
  // take whatever CUs it leaves idle, so the tile that costs the least CU time is the best one, not the
  // one that finishes first on an empty chip.
  int shared_chip;
};

// Ordered final sums of partial rows (see launch_grad_reduce below): out0[c] += sum_y p0[y][c] over `parts`
// rows of N floats, the same for the optional pair p1/out1; block0 = first workgroup of the segment.
struct GradReduceSeg { const float* p0; float* out0; const float* p1; float* out1; int N, parts, block0; };
struct GradReduceBatch { GradReduceSeg seg[8]; int n; };

// up to MAX independent GEMMs for one launch; first[p] = index of problem p's first workgroup.
// Workgroups from first[MAX] on (there are grad_reduce_blocks(tail) of them) do the reductions of `tail`.
struct GemmGroup {
  static constexpr int MAX = 4;
  GemmDesc d[MAX];
  int first[MAX + 1];
  int n;
  int whole_launch_ranges;   // 1: the XCD ranges are cut from the concatenated tile sequences of all problems
  GradReduceBatch tail;
};

// dtype: 0 fp32, 1 bf16 (enum bamboo_dtype).  All launchers return hipError_t
// from the launch and never synchronise.
hipError_t launch_gemm_simple(hipStream_t s, int dtype, const GemmDesc& d);
// bf16 MFMA path; returns hipErrorNotSupported when the shape is not covered.
hipError_t launch_gemm_mfma(hipStream_t s, const GemmDesc& d);
hipError_t launch_gemm(hipStream_t s, int dtype, const GemmDesc& d);
// one-time device tables of the MFMA GEMM (GELU lookup): filled and waited for here, at set-up
hipError_t prepare_gemm_tables(hipStream_t s);
// n independent weight-gradient GEMMs (EPI_ACC_F32): one launch where the MFMA kernel covers them all,
// otherwise one launch each
// tail (optional): reductions that depend on nothing in the group, done by extra workgroups of the same
// launch, which find idle CUs while the last GEMM tiles run; *tail_done says whether the launch took them
// (a path that does not leaves them to the caller's launch_grad_reduce).
hipError_t launch_gemm_group_mfma(hipStream_t s, const GemmDesc* d, int n, const GradReduceBatch* tail = nullptr);
hipError_t launch_gemm_group(hipStream_t s, int dtype, const GemmDesc* d, int n, const GradReduceBatch* tail = nullptr,
                             bool* tail_done = nullptr);
// output tile of the MFMA kernel: 10*WM + WN forces (64*WM) x (64*WN), 0 = automatic; returns the previous code
bool gemm_tile_code_valid(int code);
int set_gemm_tile(int code);
// LDS ring depth of the pipelined MFMA kernel: 2, 3 or 4 forces it where it fits, 0 = automatic; returns the previous value
int set_gemm_stages(int n);

// ---- attention ---------------------------------------------------------------
// qkv [T,3H] (queries | keys | values), ctx [T,H], lse fp32 [B,heads,S]
struct AttnDesc {
  int B, S, heads, d;   // H = heads*d
  int causal;
  const void* qkv;
  void* ctx;            // fwd out / bwd in
  float* lse;           // fwd out / bwd in: log-sum-exp of the scaled scores per row
  const void* dctx;     // bwd in
  void* dqkv;           // bwd out [T,3H]
  float* delta;         // bwd scratch [B,heads,S]
  // bwd, optional: dqkv_colsum (device fp32, B * ceil(S/128) rows of 3H) receives, per sample and block of
  // 128 tokens, the column sums of the dqkv rows the MFMA kernels store (the bias gradient of the QKV
  // projection, without reading dqkv again); *dqkv_colsum_parts (host) = number of rows written, left
  // untouched by a kernel that does not do it.
  float* dqkv_colsum;
  int* dqkv_colsum_parts;
};
hipError_t launch_attention_fwd_simple(hipStream_t s, int dtype, const AttnDesc& d);
hipError_t launch_attention_bwd_simple(hipStream_t s, int dtype, const AttnDesc& d);
hipError_t launch_attention_fwd_mfma(hipStream_t s, const AttnDesc& d);
hipError_t launch_attention_bwd_mfma(hipStream_t s, const AttnDesc& d);
hipError_t launch_attention_fwd(hipStream_t s, int dtype, const AttnDesc& d);
hipError_t launch_attention_bwd(hipStream_t s, int dtype, const AttnDesc& d);

// ---- LayerNorm / reductions / misc ------------------------------------------------
// y = gamma * (r - mean) * rstd + beta; stats[2*t] = mean, stats[2*t+1] = rstd
hipError_t launch_layernorm_fwd(hipStream_t s, int dtype, int T, int H, float eps, const void* r, const void* gamma,
                                const void* beta, void* y, float* stats);
// dr = LN backward(dout) (+ add if add != nullptr); dgamma/dbeta (fp32) += column sums
// partial: fp32 scratch of ln_bwd_partial_floats(H) floats
hipError_t launch_layernorm_bwd(hipStream_t s, int dtype, int T, int H, const void* dout, const void* r,
                                const float* stats, const void* gamma, const void* add, void* dr, float* dgamma,
                                float* dbeta, float* partial);
// out[n] (fp32) += sum_t a[t,n]; partial: fp32 scratch of colsum_partial_floats(N)
hipError_t launch_colsum_acc(hipStream_t s, int dtype, int T, int N, const void* a, float* out, float* partial);
// out[n] += sum over the first `parts` rows of partial[parts][N], in order
hipError_t launch_colsum_final(hipStream_t s, int N, int parts, const float* partial, float* out);
// The two halves of the calls above, for callers that batch the final sums of several reductions:
// the *_partials launchers write partial rows only (row count returned through *parts; at most
// reduce_max_partials() rows of N floats), launch_grad_reduce then adds the ordered sums of up to
// eight partial sets to their fp32 destinations in one launch.
hipError_t launch_layernorm_bwd_partials(hipStream_t s, int dtype, int T, int H, const void* dout, const void* r,
                                         const float* stats, const void* gamma, const void* add, void* dr, float* pg,
                                         float* pb, float* pc, int* parts);
hipError_t launch_colsum_partials(hipStream_t s, int dtype, int T, int N, const void* a, float* partial, int* parts);
// appends out0[c] += sum_y p0[y][c] (and the same for the optional second pair p1/out1); false when full
bool grad_reduce_add(GradReduceBatch* b, int N, int parts, const float* p0, float* out0, const float* p1, float* out1);
hipError_t launch_grad_reduce(hipStream_t s, const GradReduceBatch& b);
int grad_reduce_blocks(const GradReduceBatch& b);   // workgroups (of 64 columns each) the batch needs
size_t reduce_max_partials();
int colsum_partial_rows(int dtype, int T, int N);   // partial rows launch_colsum_partials writes for this shape
size_t colsum_partial_floats(int N);
size_t ln_bwd_partial_floats(int H);
hipError_t launch_bubble(hipStream_t s, float microseconds);

// ---- model ends (wrap-around stage) ---------------------------------------------
hipError_t launch_embed_fwd(hipStream_t s, int dtype, int T, int S, int H, int V, const int* ids, const void* Etok,
                            const void* Epos, void* out);
hipError_t launch_embed_bwd(hipStream_t s, int dtype, int T, int S, int H, int V, const int* ids, const void* g,
                            float* dEtok, float* dEpos);
hipError_t launch_xent_fwd(hipStream_t s, int dtype, int T, int V, const void* logits, const int* labels, float* lse,
                           float* loss_tok);
hipError_t launch_xent_bwd(hipStream_t s, int dtype, int T, int V, const void* logits, const int* labels,
                           const float* lse, float scale, void* dlogits);
hipError_t launch_ordered_sum(hipStream_t s, long n, const float* in, float scale, float* out);

// ---- optimizer ------------------------------------------------------------------
// Adam on n parameters (n a multiple of 4): fp32 gradient g, fp32 master weights and moments m, v
// updated in place, w = storage-dtype copy of the new master weights.  step counts from 1.
hipError_t launch_adam(hipStream_t s, int dtype, long n, const float* g, float* master, float* m, float* v, void* w,
                       float lr, float beta1, float beta2, float eps, int step);
// master[i] = (float) w[i]
hipError_t launch_widen(hipStream_t s, int dtype, long n, const void* w, float* master);
hipError_t launch_fill_zero(hipStream_t s, long n, float* p);
hipError_t launch_copy(hipStream_t s, const void* src, void* dst, size_t bytes);
hipError_t launch_calibration_copy(hipStream_t s, const void* src, void* dst, size_t bytes);

}  // namespace bamboo
