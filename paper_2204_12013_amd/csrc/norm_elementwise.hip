// LayerNorm forward/backward, column reductions (bias and gain/shift
// gradients) and the simulated-bubble kernel.  All HBM-bound: one wavefront per
// token row, 16-byte vector accesses, rows held in registers between the
// statistics pass and the output pass, wavefront reductions.  Reductions over
// tokens are two-stage with a fixed order (per-workgroup partial sums, then one
// ordered sum), so results are bitwise reproducible -- needed for FRC == FNC
// and for failover == failure-free gradients.
#include <atomic>

#include "common.h"
#include "reduce_device.h"

namespace bamboo {

template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  typedef float4 Raw;
  __device__ static __forceinline__ Raw load_raw(const float* p) { return *(const float4*)p; }
  __device__ static __forceinline__ void unpack(const Raw& t, float (&v)[4]) { v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w; }
  __device__ static __forceinline__ void load(const float* p, float (&v)[4]) {
    const float4 t = *(const float4*)p;
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  __device__ static __forceinline__ void store(float* p, const float (&v)[4]) {
    *(float4*)p = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  typedef __attribute__((ext_vector_type(8))) __bf16 raw;
  typedef raw Raw;
  __device__ static __forceinline__ Raw load_raw(const bf16_t* p) { return *(const raw*)p; }
  __device__ static __forceinline__ void unpack(const Raw& t, float (&v)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
  }
  __device__ static __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const raw t = *(const raw*)p;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
  }
  __device__ static __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    raw t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = (bf16_t)v[i];
    *(raw*)p = t;
  }
};

constexpr int kMaxPartials = 256;   // workgroups contributing partial column sums

// ------------------------------------------------------------ LayerNorm forward
// NCH = vector chunks a lane keeps in registers (row length <= NCH * 64 * V).  Every load of a
// row is requested before the first is used (lanes past the row's end re-read its last vector and
// drop it), so a wavefront keeps the whole row in flight.
template <typename T, int NCH>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(int T_rows, int H, float eps, const T* __restrict__ r,
                                                            const T* __restrict__ gamma, const T* __restrict__ beta,
                                                            T* __restrict__ y, float* __restrict__ stats) {
  constexpr int V = Vec<T>::N;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T_rows) return;
  const T* rr = r + (long)row * H;
  const int nvec = H / V;
  typename Vec<T>::Raw raw[NCH], graw[NCH], braw[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) raw[j] = Vec<T>::load_raw(rr + min(lane + 64 * j, nvec - 1) * V);
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    graw[j] = Vec<T>::load_raw(gamma + min(lane + 64 * j, nvec - 1) * V);
    braw[j] = Vec<T>::load_raw(beta + min(lane + 64 * j, nvec - 1) * V);
  }
  float v[NCH][V];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    Vec<T>::unpack(raw[j], v[j]);
    const float keep = lane + 64 * j < nvec ? 1.f : 0.f;
#pragma unroll
    for (int i = 0; i < V; ++i) s += keep * v[j][i];
  }
  const float mean = wave_sum(s) / (float)H;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const float keep = lane + 64 * j < nvec ? 1.f : 0.f;
#pragma unroll
    for (int i = 0; i < V; ++i) q += keep * (v[j][i] - mean) * (v[j][i] - mean);
  }
  const float rstd = rsqrtf(wave_sum(q) / (float)H + eps);
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = lane + 64 * j;
    float g[V], b[V], o[V];
    Vec<T>::unpack(graw[j], g);
    Vec<T>::unpack(braw[j], b);
#pragma unroll
    for (int i = 0; i < V; ++i) o[i] = g[i] * ((v[j][i] - mean) * rstd) + b[i];
    if (c < nvec) Vec<T>::store(y + (long)row * H + c * V, o);
  }
  if (lane == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
}

// any row length: three passes over the row (the later ones hit L2)
template <typename T>
__global__ __launch_bounds__(256) void layernorm_fwd_long_kernel(int T_rows, int H, float eps, const T* __restrict__ r,
                                                                 const T* __restrict__ gamma,
                                                                 const T* __restrict__ beta, T* __restrict__ y,
                                                                 float* __restrict__ stats) {
  constexpr int V = Vec<T>::N;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T_rows) return;
  const T* rr = r + (long)row * H;
  const int nvec = H / V;
  float s = 0.f;
  for (int c = lane; c < nvec; c += 64) {
    float v[V];
    Vec<T>::load(rr + c * V, v);
#pragma unroll
    for (int i = 0; i < V; ++i) s += v[i];
  }
  const float mean = wave_sum(s) / (float)H;
  float q = 0.f;
  for (int c = lane; c < nvec; c += 64) {
    float v[V];
    Vec<T>::load(rr + c * V, v);
#pragma unroll
    for (int i = 0; i < V; ++i) q += (v[i] - mean) * (v[i] - mean);
  }
  const float rstd = rsqrtf(wave_sum(q) / (float)H + eps);
  for (int c = lane; c < nvec; c += 64) {
    float v[V], g[V], b[V], o[V];
    Vec<T>::load(rr + c * V, v);
    Vec<T>::load(gamma + c * V, g);
    Vec<T>::load(beta + c * V, b);
#pragma unroll
    for (int i = 0; i < V; ++i) o[i] = g[i] * ((v[i] - mean) * rstd) + b[i];
    Vec<T>::store(y + (long)row * H + c * V, o);
  }
  if (lane == 0) {
    stats[2 * row] = mean;
    stats[2 * row + 1] = rstd;
  }
}

template <typename T>
static hipError_t ln_fwd_impl(hipStream_t s, int T_rows, int H, float eps, const void* r, const void* gamma,
                              const void* beta, void* y, float* stats) {
  constexpr int V = Vec<T>::N;
  dim3 grid((T_rows + 3) / 4);
  const int nch = (H / V + 63) / 64;
#define LN_FWD(K)                                                                                              \
  hipLaunchKernelGGL(K, grid, dim3(256), 0, s, T_rows, H, eps, (const T*)r, (const T*)gamma, (const T*)beta, \
                     (T*)y, stats)
  if (nch <= 1) LN_FWD((layernorm_fwd_kernel<T, 1>));
  else if (nch <= 2) LN_FWD((layernorm_fwd_kernel<T, 2>));
  else if (nch <= 4) LN_FWD((layernorm_fwd_kernel<T, 4>));
  else if (nch <= 8) LN_FWD((layernorm_fwd_kernel<T, 8>));
  else LN_FWD(layernorm_fwd_long_kernel<T>);
#undef LN_FWD
  return hipGetLastError();
}

hipError_t launch_layernorm_fwd(hipStream_t s, int dtype, int T, int H, float eps, const void* r, const void* gamma,
                                const void* beta, void* y, float* stats) {
  return dtype == 0 ? ln_fwd_impl<float>(s, T, H, eps, r, gamma, beta, y, stats)
                    : ln_fwd_impl<bf16_t>(s, T, H, eps, r, gamma, beta, y, stats);
}

// ----------------------------------------------------------- LayerNorm backward
// dr = (dhat - mean(dhat) - rhat * mean(dhat * rhat)) * rstd, dhat = dout * gamma.
// Fused variant: the workgroup also accumulates its rows' contributions to the
// gain and shift gradients (sum dout*rhat, sum dout) and, if COLSUM, the column sums of the stored
// output dr (the bias gradient of the linear layer whose output gradient dr is), and writes one
// partial row of each per workgroup; lane-owned columns stay in registers across rows.
// A wavefront takes two of its rows per pass and requests all of their data before it works on
// either: the kernel is bound by memory latency times bytes in flight, not by arithmetic.  Lanes
// past the row's end re-read its last vector and zero it.
template <typename T, int NCH, bool ADD, bool COLSUM>
__global__ __launch_bounds__(256) void layernorm_bwd_fused_kernel(int T_rows, int H, int rows_per_block,
                                                                  const T* __restrict__ dout, const T* __restrict__ r,
                                                                  const float* __restrict__ stats,
                                                                  const T* __restrict__ gamma,
                                                                  const T* __restrict__ add, T* __restrict__ dr,
                                                                  float* __restrict__ pg, float* __restrict__ pb,
                                                                  float* __restrict__ pc) {
  constexpr int V = Vec<T>::N;
  typedef typename Vec<T>::Raw Raw;
  extern __shared__ float red[];                 // [4][H]
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int nvec = H / V;
  float g[NCH][V], ag[NCH][V], ab[NCH][V], ac[COLSUM ? NCH : 1][V];
  int cc[NCH];
  float keep[NCH];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int c = lane + 64 * j;
    cc[j] = min(c, nvec - 1) * V;
    keep[j] = c < nvec ? 1.f : 0.f;
#pragma unroll
    for (int i = 0; i < V; ++i) { ag[j][i] = 0.f; ab[j][i] = 0.f; }
    if (COLSUM) {
#pragma unroll
      for (int i = 0; i < V; ++i) ac[j][i] = 0.f;
    }
    Vec<T>::load(gamma + cc[j], g[j]);
  }
  const int row_end = min(T_rows, (int)(blockIdx.x + 1) * rows_per_block);
  for (int row0 = blockIdx.x * rows_per_block + w; row0 < row_end; row0 += 8) {
    // second row of the pass: if there is none, the first is read again and its results dropped
    const bool two = row0 + 4 < row_end;
    const int rows[2] = {row0, two ? row0 + 4 : row0};
    Raw dw[2][NCH], xw[2][NCH], aw[2][ADD ? NCH : 1];
    float mean[2], rstd[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const long off = (long)rows[u] * H;
      mean[u] = stats[2 * rows[u]];
      rstd[u] = stats[2 * rows[u] + 1];
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        dw[u][j] = Vec<T>::load_raw(dout + off + cc[j]);
        xw[u][j] = Vec<T>::load_raw(r + off + cc[j]);
        if (ADD) aw[u][j] = Vec<T>::load_raw(add + off + cc[j]);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const float use = (u == 0 || two) ? 1.f : 0.f;
      const long off = (long)rows[u] * H;
      float d[NCH][V], xh[NCH][V];
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        float x[V];
        Vec<T>::unpack(dw[u][j], d[j]);
        Vec<T>::unpack(xw[u][j], x);
        const float k = keep[j] * use;
#pragma unroll
        for (int i = 0; i < V; ++i) {
          d[j][i] *= k;
          xh[j][i] = (x[i] - mean[u]) * rstd[u];
          ag[j][i] += d[j][i] * xh[j][i];
          ab[j][i] += d[j][i];
          d[j][i] *= g[j][i];                      // dhat
          s1 += d[j][i];
          s2 += d[j][i] * xh[j][i];
        }
      }
      const float m1 = wave_sum(s1) / (float)H;
      const float m2 = wave_sum(s2) / (float)H;
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        float o[V];
#pragma unroll
        for (int i = 0; i < V; ++i) o[i] = (d[j][i] - m1 - xh[j][i] * m2) * rstd[u];
        if (ADD) {
          float a[V];
          Vec<T>::unpack(aw[u][j], a);
#pragma unroll
          for (int i = 0; i < V; ++i) o[i] += a[i];
        }
        if (COLSUM) {
          const float k = keep[j] * use;
#pragma unroll
          for (int i = 0; i < V; ++i) ac[j][i] += k * round_storage<T>(o[i]);
        }
        if (lane + 64 * j < nvec && (u == 0 || two)) Vec<T>::store(dr + off + cc[j], o);
      }
    }
  }
  // ordered reduction of the four wavefronts: gain gradient, shift gradient, output column sums
#pragma unroll
  for (int which = 0; which < (COLSUM ? 3 : 2); ++which) {
    __syncthreads();
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int c = lane + 64 * j;
      if (c < nvec) {
#pragma unroll
        for (int i = 0; i < V; ++i)
          red[w * H + c * V + i] = which == 0 ? ag[j][i] : (which == 1 ? ab[j][i] : ac[COLSUM ? j : 0][i]);
      }
    }
    __syncthreads();
    float* out = (which == 0 ? pg : (which == 1 ? pb : pc)) + (long)blockIdx.x * H;
    for (int c = threadIdx.x; c < H; c += 256) out[c] = ((red[c] + red[H + c]) + red[2 * H + c]) + red[3 * H + c];
  }
}

// dr only (any row length); gain/shift gradients come from colreduce_kernel<.,1>
template <typename T>
__global__ __launch_bounds__(256) void layernorm_bwd_kernel(int T_rows, int H, const T* __restrict__ dout,
                                                            const T* __restrict__ r, const float* __restrict__ stats,
                                                            const T* __restrict__ gamma, const T* __restrict__ add,
                                                            T* __restrict__ dr) {
  constexpr int V = Vec<T>::N;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T_rows) return;
  const long off = (long)row * H;
  const float mean = stats[2 * row], rstd = stats[2 * row + 1];
  const int nvec = H / V;
  float s1 = 0.f, s2 = 0.f;
  for (int c = lane; c < nvec; c += 64) {
    float d[V], x[V], g[V];
    Vec<T>::load(dout + off + c * V, d);
    Vec<T>::load(r + off + c * V, x);
    Vec<T>::load(gamma + c * V, g);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const float dh = d[i] * g[i];
      s1 += dh;
      s2 += dh * ((x[i] - mean) * rstd);
    }
  }
  const float m1 = wave_sum(s1) / (float)H;
  const float m2 = wave_sum(s2) / (float)H;
  for (int c = lane; c < nvec; c += 64) {
    float d[V], x[V], g[V], o[V];
    Vec<T>::load(dout + off + c * V, d);
    Vec<T>::load(r + off + c * V, x);
    Vec<T>::load(gamma + c * V, g);
#pragma unroll
    for (int i = 0; i < V; ++i) o[i] = (d[i] * g[i] - m1 - (x[i] - mean) * rstd * m2) * rstd;
    if (add != nullptr) {
      float a[V];
      Vec<T>::load(add + off + c * V, a);
#pragma unroll
      for (int i = 0; i < V; ++i) o[i] += a[i];
    }
    Vec<T>::store(dr + off + c * V, o);
  }
}

// ------------------------------------------------------------ column reductions
// A workgroup covers 64*V columns (one 16-byte vector per lane) and a contiguous
// range of rows, interleaved over its four wavefronts.
// MODE 0: p0[y][c] = sum a[t,c]
// MODE 1: p0 = sum a[t,c] * rhat[t,c] (gain gradient), p1 = sum a[t,c] (shift gradient)
template <typename T, int MODE>
__global__ __launch_bounds__(256) void colreduce_kernel(int T_rows, int N, int rows_per_block,
                                                        const T* __restrict__ a, const T* __restrict__ r,
                                                        const float* __restrict__ stats, float* __restrict__ p0,
                                                        float* __restrict__ p1) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[2][4][64 * V];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = (blockIdx.x * 64 + lane) * V;
  float s0[V], s1[V];
#pragma unroll
  for (int i = 0; i < V; ++i) { s0[i] = 0.f; s1[i] = 0.f; }
  if (c < N) {
    const int row_end = min(T_rows, (int)(blockIdx.y + 1) * rows_per_block);
#pragma unroll 4
    for (int t = blockIdx.y * rows_per_block + w; t < row_end; t += 4) {
      float v[V];
      Vec<T>::load(a + (long)t * N + c, v);
      if (MODE == 0) {
#pragma unroll
        for (int i = 0; i < V; ++i) s0[i] += v[i];
      } else {
        float x[V];
        Vec<T>::load(r + (long)t * N + c, x);
        const float mean = stats[2 * t], rstd = stats[2 * t + 1];
#pragma unroll
        for (int i = 0; i < V; ++i) {
          s0[i] += v[i] * ((x[i] - mean) * rstd);
          s1[i] += v[i];
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < V; ++i) {
    red[0][w][lane * V + i] = s0[i];
    if (MODE == 1) red[1][w][lane * V + i] = s1[i];
  }
  __syncthreads();
  for (int j = threadIdx.x; j < 64 * V; j += 256) {
    const int col = blockIdx.x * 64 * V + j;
    if (col < N) {
      p0[(long)blockIdx.y * N + col] = ((red[0][0][j] + red[0][1][j]) + red[0][2][j]) + red[0][3][j];
      if (MODE == 1) p1[(long)blockIdx.y * N + col] = ((red[1][0][j] + red[1][1][j]) + red[1][2][j]) + red[1][3][j];
    }
  }
}

// out[c] += sum_y p[y][c]: 16 wavefronts each sum a contiguous sixteenth of the
// partial rows in order, then the sixteen sums are added in order.
constexpr int kFinalWaves = 16;
__global__ __launch_bounds__(1024) void colreduce_final_kernel(int N, int splits, const float* __restrict__ p0,
                                                               float* __restrict__ out0,
                                                               const float* __restrict__ p1,
                                                               float* __restrict__ out1) {
  __shared__ float red[2][kFinalWaves][64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  const int per = (splits + kFinalWaves - 1) / kFinalWaves;
  float s = 0.f, q = 0.f;
  if (c < N) {
    const int y_end = min(splits, (w + 1) * per);
#pragma unroll 8
    for (int y = w * per; y < y_end; ++y) s += p0[(long)y * N + c];
    if (p1 != nullptr) {
#pragma unroll 8
      for (int y = w * per; y < y_end; ++y) q += p1[(long)y * N + c];
    }
  }
  red[0][w][lane] = s;
  red[1][w][lane] = q;
  __syncthreads();
  if (w == 0 && c < N) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int k = 0; k < kFinalWaves; ++k) {
      a += red[0][k][lane];
      b += red[1][k][lane];
    }
    out0[c] += a;
    if (p1 != nullptr) out1[c] += b;
  }
}

// The same ordered final sum for up to eight reductions in one launch (the parameter-gradient
// reductions of one layer's backward): workgroup b serves the segment whose block range holds b.
__global__ __launch_bounds__(1024) void colreduce_final_batch_kernel(GradReduceBatch batch) {
  __shared__ float red[kReduceLdsFloats];
  colreduce_batch_block(batch, (int)blockIdx.x, red);
}

bool grad_reduce_add(GradReduceBatch* b, int N, int parts, const float* p0, float* out0, const float* p1, float* out1) {
  if (b->n >= 8) return false;
  GradReduceSeg& sg = b->seg[b->n];
  sg.p0 = p0; sg.out0 = out0; sg.p1 = p1; sg.out1 = out1; sg.N = N; sg.parts = parts;
  sg.block0 = b->n == 0 ? 0 : b->seg[b->n - 1].block0 + (b->seg[b->n - 1].N + 63) / 64;
  ++b->n;
  return true;
}
int grad_reduce_blocks(const GradReduceBatch& b) {
  return b.n <= 0 ? 0 : b.seg[b.n - 1].block0 + (b.seg[b.n - 1].N + 63) / 64;
}
hipError_t launch_grad_reduce(hipStream_t s, const GradReduceBatch& b) {
  if (b.n <= 0) return hipSuccess;
  static_assert(kReduceGroups == kFinalWaves, "one group of partial rows per wavefront");
  const int blocks = grad_reduce_blocks(b);
  hipLaunchKernelGGL(colreduce_final_batch_kernel, dim3(blocks), dim3(1024), 0, s, b);
  return hipGetLastError();
}

// rows per workgroup and number of workgroups along the token axis
static void split_rows(int T, int max_blocks, int* rows_per_block, int* blocks) {
  int rpb = (T + max_blocks - 1) / max_blocks;
  if (rpb < 4) rpb = 4;
  *rows_per_block = rpb;
  *blocks = (T + rpb - 1) / rpb;
}
hipError_t launch_colsum_final(hipStream_t s, int N, int parts, const float* partial, float* out) {
  hipLaunchKernelGGL(colreduce_final_kernel, dim3((N + 63) / 64), dim3(1024), 0, s, N, parts, partial, out,
                     (const float*)nullptr, (float*)nullptr);
  return hipGetLastError();
}
size_t reduce_max_partials() { return kMaxPartials; }
size_t colsum_partial_floats(int N) { return (size_t)kMaxPartials * N; }
size_t ln_bwd_partial_floats(int H) { return (size_t)2 * kMaxPartials * H; }

// launch shape of the column-sum kernel: workgroups across the columns (64 vectors of V each), rows per
// workgroup and workgroups along the token axis (= partial rows written)
static void colsum_shape(int V, int T_rows, int N, int* col_blocks, int* rows_per_block, int* row_blocks) {
  *col_blocks = (N + 64 * V - 1) / (64 * V);
  int max_blocks = 512 / *col_blocks;           // about two workgroups per CU in total
  if (max_blocks > kMaxPartials) max_blocks = kMaxPartials;
  if (max_blocks < 1) max_blocks = 1;
  split_rows(T_rows, max_blocks, rows_per_block, row_blocks);
}
int colsum_partial_rows(int dtype, int T, int N) {
  int cb, rpb, rb;
  colsum_shape(dtype == 0 ? Vec<float>::N : Vec<bf16_t>::N, T, N, &cb, &rpb, &rb);
  return rb;
}

template <typename T>
static hipError_t colsum_partials_impl(hipStream_t s, int T_rows, int N, const void* a, float* partial, int* parts) {
  constexpr int V = Vec<T>::N;
  int col_blocks, rpb, rb;
  colsum_shape(V, T_rows, N, &col_blocks, &rpb, &rb);
  hipLaunchKernelGGL((colreduce_kernel<T, 0>), dim3(col_blocks, rb), dim3(256), 0, s, T_rows, N, rpb, (const T*)a,
                     (const T*)nullptr, (const float*)nullptr, partial, (float*)nullptr);
  *parts = rb;
  return hipGetLastError();
}

hipError_t launch_colsum_partials(hipStream_t s, int dtype, int T, int N, const void* a, float* partial, int* parts) {
  return dtype == 0 ? colsum_partials_impl<float>(s, T, N, a, partial, parts)
                    : colsum_partials_impl<bf16_t>(s, T, N, a, partial, parts);
}

hipError_t launch_colsum_acc(hipStream_t s, int dtype, int T, int N, const void* a, float* out, float* partial) {
  int parts = 0;
  const hipError_t e = launch_colsum_partials(s, dtype, T, N, a, partial, &parts);
  if (e != hipSuccess) return e;
  return launch_colsum_final(s, N, parts, partial, out);
}

// dr and the partial rows of the gain / shift gradients (pg, pb: kMaxPartials x H floats each) and,
// if pc != nullptr, of the column sums of dr; the number of partial rows written comes back in *parts
template <typename T>
static hipError_t ln_bwd_partials_impl(hipStream_t s, int T_rows, int H, const void* dout, const void* r,
                                       const float* stats, const void* gamma, const void* add, void* dr, float* pg,
                                       float* pb, float* pc, int* parts) {
  constexpr int V = Vec<T>::N;
  const int nch = (H / V + 63) / 64;
  int rpb, rb;
  if (nch <= 4 && (size_t)4 * H * sizeof(float) <= 48 * 1024) {
    split_rows(T_rows, kMaxPartials, &rpb, &rb);
    const size_t sh = (size_t)4 * H * sizeof(float);
#define LN_BWD1(NC, A, C)                                                                                          \
  hipLaunchKernelGGL((layernorm_bwd_fused_kernel<T, NC, A, C>), dim3(rb), dim3(256), sh, s, T_rows, H, rpb,         \
                     (const T*)dout, (const T*)r, stats, (const T*)gamma, (const T*)add, (T*)dr, pg, pb, pc)
#define LN_BWD(NC)                                                                                                 \
  do {                                                                                                             \
    if (add != nullptr) { if (pc != nullptr) LN_BWD1(NC, true, true); else LN_BWD1(NC, true, false); }             \
    else { if (pc != nullptr) LN_BWD1(NC, false, true); else LN_BWD1(NC, false, false); }                          \
  } while (0)
    if (nch <= 1) LN_BWD(1);
    else if (nch <= 2) LN_BWD(2);
    else LN_BWD(4);
#undef LN_BWD1
#undef LN_BWD
  } else {
    const int col_blocks = (H + 64 * V - 1) / (64 * V);
    int max_blocks = 512 / col_blocks;
    if (max_blocks > kMaxPartials) max_blocks = kMaxPartials;
    if (max_blocks < 1) max_blocks = 1;
    split_rows(T_rows, max_blocks, &rpb, &rb);
    hipLaunchKernelGGL((colreduce_kernel<T, 1>), dim3(col_blocks, rb), dim3(256), 0, s, T_rows, H, rpb, (const T*)dout,
                       (const T*)r, stats, pg, pb);
    hipLaunchKernelGGL(layernorm_bwd_kernel<T>, dim3((T_rows + 3) / 4), dim3(256), 0, s, T_rows, H, (const T*)dout,
                       (const T*)r, stats, (const T*)gamma, (const T*)add, (T*)dr);
    if (pc != nullptr)   // same row split, so all three partial sets have rb rows
      hipLaunchKernelGGL((colreduce_kernel<T, 0>), dim3(col_blocks, rb), dim3(256), 0, s, T_rows, H, rpb,
                         (const T*)dr, (const T*)nullptr, (const float*)nullptr, pc, (float*)nullptr);
  }
  *parts = rb;
  return hipGetLastError();
}

hipError_t launch_layernorm_bwd_partials(hipStream_t s, int dtype, int T, int H, const void* dout, const void* r,
                                         const float* stats, const void* gamma, const void* add, void* dr, float* pg,
                                         float* pb, float* pc, int* parts) {
  return dtype == 0 ? ln_bwd_partials_impl<float>(s, T, H, dout, r, stats, gamma, add, dr, pg, pb, pc, parts)
                    : ln_bwd_partials_impl<bf16_t>(s, T, H, dout, r, stats, gamma, add, dr, pg, pb, pc, parts);
}

hipError_t launch_layernorm_bwd(hipStream_t s, int dtype, int T, int H, const void* dout, const void* r,
                                const float* stats, const void* gamma, const void* add, void* dr, float* dgamma,
                                float* dbeta, float* partial) {
  float* p0 = partial;
  float* p1 = partial + (size_t)kMaxPartials * H;
  int parts = 0;
  const hipError_t e =
      launch_layernorm_bwd_partials(s, dtype, T, H, dout, r, stats, gamma, add, dr, p0, p1, nullptr, &parts);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colreduce_final_kernel, dim3((H + 63) / 64), dim3(1024), 0, s, H, parts, p0, dgamma, p1, dbeta);
  return hipGetLastError();
}

// --------------------------------------------------------------------- copy
// Plain 16-byte-per-lane copy. The replica sync uses copy_kernel; the copy of a
// known size that the HBM traffic counters of the other kernels are scaled by
// has a kernel name of its own, so that a counter summary can tell it apart.
__device__ __forceinline__ void copy_body(const float4* __restrict__ src, float4* __restrict__ dst, long n16) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n16; i += (long)gridDim.x * 256) dst[i] = src[i];
}
__global__ __launch_bounds__(256) void copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, long n16) {
  copy_body(src, dst, n16);
}
__global__ __launch_bounds__(256) void calibration_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                               long n16) {
  copy_body(src, dst, n16);
}
static hipError_t launch_copy_impl(hipStream_t s, const void* src, void* dst, size_t bytes, bool calibration) {
  const long n16 = (long)(bytes / 16);
  if (n16 == 0) return hipSuccess;
  long blocks = (n16 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (calibration)
    hipLaunchKernelGGL(calibration_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const float4*)src, (float4*)dst, n16);
  else
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const float4*)src, (float4*)dst, n16);
  return hipGetLastError();
}
hipError_t launch_copy(hipStream_t s, const void* src, void* dst, size_t bytes) {
  return launch_copy_impl(s, src, dst, bytes, false);
}
hipError_t launch_calibration_copy(hipStream_t s, const void* src, void* dst, size_t bytes) {
  return launch_copy_impl(s, src, dst, bytes, true);
}

// ------------------------------------------------------------------- bubble
// One wavefront waits on the constant-rate device clock.  The wait always ends:
// the clock advances on its own, and an iteration cap bounds it regardless.
__global__ void bubble_kernel(long long clock_ticks, int* sink) {
  const long long t0 = wall_clock64();
  long long it = 0;
  while (wall_clock64() - t0 < clock_ticks && it < (1LL << 34)) {
    __builtin_amdgcn_s_sleep(32);
    ++it;
  }
  if (sink != nullptr && it < 0) *sink = (int)it;  // never taken; keeps the loop observable
}

hipError_t launch_bubble(hipStream_t s, float microseconds) {
  // the device clock rate, read once (racing first calls read the same value: the store is atomic)
  static std::atomic<int> rate_cache{0};
  int rate_khz = rate_cache.load();
  if (rate_khz == 0) {
    int dev = 0, r = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
    if (hipDeviceGetAttribute(&r, hipDeviceAttributeWallClockRate, dev) != hipSuccess || r <= 0) r = 100000;
    rate_cache.store(r);
    rate_khz = r;
  }
  if (microseconds <= 0.f) return hipSuccess;
  if (microseconds > 5e6f) microseconds = 5e6f;
  const long long ticks = (long long)((double)microseconds * 1e-3 * (double)rate_khz);
  hipLaunchKernelGGL(bubble_kernel, dim3(1), dim3(64), 0, s, ticks, (int*)nullptr);
  return hipGetLastError();
}

}  // namespace bamboo
