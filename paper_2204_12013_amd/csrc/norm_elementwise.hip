// LayerNorm forward/backward, column reductions (bias and gain/shift
// gradients) and the simulated-bubble kernel.  All HBM-bound: one wavefront per
// token row, 16-byte vector loads, wavefront reductions; the later passes over a
// row hit L2.  Reductions over tokens are two-stage with a fixed order, so the
// results are bitwise reproducible (needed for FRC == FNC and for
// failover == failure-free gradients).
#include "common.h"

namespace bamboo {

template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  typedef float4 raw;
  __device__ static void load(const float* p, float (&v)[4]) {
    const float4 t = *(const float4*)p;
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
  __device__ static void store(float* p, const float (&v)[4]) { *(float4*)p = make_float4(v[0], v[1], v[2], v[3]); }
};
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  typedef __attribute__((ext_vector_type(8))) __bf16 raw;
  __device__ static void load(const bf16_t* p, float (&v)[8]) {
    const raw t = *(const raw*)p;
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = (float)t[i];
  }
  __device__ static void store(bf16_t* p, const float (&v)[8]) {
    raw t;
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = (bf16_t)v[i];
    *(raw*)p = t;
  }
};

// ------------------------------------------------------------ LayerNorm forward
template <typename T>
__global__ __launch_bounds__(256) void layernorm_fwd_kernel(int T_rows, int H, float eps, const T* __restrict__ r,
                                                            const T* __restrict__ gamma, const T* __restrict__ beta,
                                                            T* __restrict__ y, float* __restrict__ stats) {
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

hipError_t launch_layernorm_fwd(hipStream_t s, int dtype, int T, int H, float eps, const void* r, const void* gamma,
                                const void* beta, void* y, float* stats) {
  dim3 grid((T + 3) / 4);
  if (dtype == 0)
    hipLaunchKernelGGL(layernorm_fwd_kernel<float>, grid, dim3(256), 0, s, T, H, eps, (const float*)r,
                       (const float*)gamma, (const float*)beta, (float*)y, stats);
  else
    hipLaunchKernelGGL(layernorm_fwd_kernel<bf16_t>, grid, dim3(256), 0, s, T, H, eps, (const bf16_t*)r,
                       (const bf16_t*)gamma, (const bf16_t*)beta, (bf16_t*)y, stats);
  return hipGetLastError();
}

// ----------------------------------------------------------- LayerNorm backward
// dr = (dhat - mean(dhat) - rhat * mean(dhat * rhat)) * rstd, dhat = dout * gamma
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
// MODE 0: p0[y][c] = sum over the block's rows of a[t,c]
// MODE 1: p0 = sum a[t,c] * rhat[t,c] (gain gradient), p1 = sum a[t,c] (shift gradient)
constexpr int kRowSplits = 32;

template <typename T, int MODE>
__global__ __launch_bounds__(256) void colreduce_kernel(int T_rows, int N, const T* __restrict__ a,
                                                        const T* __restrict__ r, const float* __restrict__ stats,
                                                        float* __restrict__ p0, float* __restrict__ p1) {
  __shared__ float red[4][2][128];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = blockIdx.x * 128 + lane * 2;
  float s0[2] = {0.f, 0.f}, s1[2] = {0.f, 0.f};
  if (c < N) {
    for (int t = blockIdx.y * 4 + w; t < T_rows; t += gridDim.y * 4) {
      const long i = (long)t * N + c;
      const float a0 = to_f32<T>(a[i]), a1 = to_f32<T>(a[i + 1]);
      if (MODE == 0) {
        s0[0] += a0;
        s0[1] += a1;
      } else {
        const float mean = stats[2 * t], rstd = stats[2 * t + 1];
        s0[0] += a0 * ((to_f32<T>(r[i]) - mean) * rstd);
        s0[1] += a1 * ((to_f32<T>(r[i + 1]) - mean) * rstd);
        s1[0] += a0;
        s1[1] += a1;
      }
    }
  }
  red[w][0][lane * 2] = s0[0];
  red[w][0][lane * 2 + 1] = s0[1];
  red[w][1][lane * 2] = s1[0];
  red[w][1][lane * 2 + 1] = s1[1];
  __syncthreads();
  if (w == 0 && c < N) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int cc = lane * 2 + j;
      p0[(long)blockIdx.y * N + c + j] = ((red[0][0][cc] + red[1][0][cc]) + red[2][0][cc]) + red[3][0][cc];
      if (MODE == 1)
        p1[(long)blockIdx.y * N + c + j] = ((red[0][1][cc] + red[1][1][cc]) + red[2][1][cc]) + red[3][1][cc];
    }
  }
}

// out[c] += sum_y p[y][c] in the fixed order y = 0, 1, ...
__global__ void colreduce_final_kernel(int N, int splits, const float* __restrict__ p0, float* __restrict__ out0,
                                       const float* __restrict__ p1, float* __restrict__ out1) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= N) return;
  float s = 0.f;
  for (int y = 0; y < splits; ++y) s += p0[(long)y * N + c];
  out0[c] += s;
  if (p1 != nullptr) {
    float q = 0.f;
    for (int y = 0; y < splits; ++y) q += p1[(long)y * N + c];
    out1[c] += q;
  }
}

static int row_splits(int T) {
  int s = (T + 3) / 4;
  return s < kRowSplits ? (s < 1 ? 1 : s) : kRowSplits;
}
size_t colsum_partial_floats(int N) { return (size_t)kRowSplits * N; }
size_t ln_bwd_partial_floats(int H) { return (size_t)2 * kRowSplits * H; }

hipError_t launch_colsum_acc(hipStream_t s, int dtype, int T, int N, const void* a, float* out, float* partial) {
  const int rs = row_splits(T);
  dim3 grid((N + 127) / 128, rs);
  if (dtype == 0)
    hipLaunchKernelGGL((colreduce_kernel<float, 0>), grid, dim3(256), 0, s, T, N, (const float*)a, (const float*)nullptr,
                       (const float*)nullptr, partial, (float*)nullptr);
  else
    hipLaunchKernelGGL((colreduce_kernel<bf16_t, 0>), grid, dim3(256), 0, s, T, N, (const bf16_t*)a,
                       (const bf16_t*)nullptr, (const float*)nullptr, partial, (float*)nullptr);
  hipLaunchKernelGGL(colreduce_final_kernel, dim3((N + 255) / 256), dim3(256), 0, s, N, rs, partial, out,
                     (const float*)nullptr, (float*)nullptr);
  return hipGetLastError();
}

hipError_t launch_layernorm_bwd(hipStream_t s, int dtype, int T, int H, const void* dout, const void* r,
                                const float* stats, const void* gamma, const void* add, void* dr, float* dgamma,
                                float* dbeta, float* partial) {
  const int rs = row_splits(T);
  dim3 grid((T + 3) / 4);
  dim3 cgrid((H + 127) / 128, rs);
  float* p0 = partial;
  float* p1 = partial + (size_t)kRowSplits * H;
  if (dtype == 0) {
    hipLaunchKernelGGL((colreduce_kernel<float, 1>), cgrid, dim3(256), 0, s, T, H, (const float*)dout, (const float*)r,
                       stats, p0, p1);
    hipLaunchKernelGGL(layernorm_bwd_kernel<float>, grid, dim3(256), 0, s, T, H, (const float*)dout, (const float*)r,
                       stats, (const float*)gamma, (const float*)add, (float*)dr);
  } else {
    hipLaunchKernelGGL((colreduce_kernel<bf16_t, 1>), cgrid, dim3(256), 0, s, T, H, (const bf16_t*)dout,
                       (const bf16_t*)r, stats, p0, p1);
    hipLaunchKernelGGL(layernorm_bwd_kernel<bf16_t>, grid, dim3(256), 0, s, T, H, (const bf16_t*)dout,
                       (const bf16_t*)r, stats, (const bf16_t*)gamma, (const bf16_t*)add, (bf16_t*)dr);
  }
  hipLaunchKernelGGL(colreduce_final_kernel, dim3((H + 255) / 256), dim3(256), 0, s, H, rs, p0, dgamma, p1, dbeta);
  return hipGetLastError();
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
  static int rate_khz = 0;
  if (rate_khz == 0) {
    int dev = 0, r = 0;
    if (hipGetDevice(&dev) != hipSuccess) return hipGetLastError();
    if (hipDeviceGetAttribute(&r, hipDeviceAttributeWallClockRate, dev) != hipSuccess || r <= 0) r = 100000;
    rate_khz = r;
  }
  if (microseconds <= 0.f) return hipSuccess;
  if (microseconds > 5e6f) microseconds = 5e6f;
  const long long ticks = (long long)((double)microseconds * 1e-3 * (double)rate_khz);
  hipLaunchKernelGGL(bubble_kernel, dim3(1), dim3(64), 0, s, ticks, (int*)nullptr);
  return hipGetLastError();
}

}  // namespace bamboo
