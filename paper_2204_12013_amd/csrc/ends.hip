// Kernels of the two ends of the model, which only the wrap-around stage touches
// (Section 5.1: the last node holds the replica of the first node's layers and
// fetches the input samples itself): token + position embedding and its
// gradient at the front, softmax cross-entropy over the LM head's logits at the
// back.  All HBM-bound; no atomics -- a table row that several tokens hit is
// summed by the workgroup of its first occurrence, in token order.
#include <math.h>

#include "common.h"

namespace bamboo {

namespace {

template <typename T> struct V8 { typedef T type __attribute__((ext_vector_type(8))); };

__device__ __forceinline__ int clamp_id(int id, int V) { return id < 0 ? 0 : (id >= V ? V - 1 : id); }

// out[t,:] = E_tok[ids[t],:] + E_pos[t mod S,:]; one wave per token, 16-byte (bf16) accesses
template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(int Tn, int S, int H, int V, const int* __restrict__ ids,
                                                        const T* __restrict__ Etok, const T* __restrict__ Epos,
                                                        T* __restrict__ out) {
  typedef typename V8<T>::type vec;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= Tn) return;
  const int lane = threadIdx.x & 63;
  const T* a = Etok + (long)clamp_id(ids[t], V) * H;
  const T* b = Epos + (long)(t % S) * H;
  T* o = out + (long)t * H;
  for (int c = lane * 8; c < H; c += 512) {
    const vec va = *(const vec*)(a + c), vb = *(const vec*)(b + c);
    vec vo;
#pragma unroll
    for (int j = 0; j < 8; ++j) vo[j] = from_f32<T>(to_f32<T>(va[j]) + to_f32<T>(vb[j]));
    *(vec*)(o + c) = vo;
  }
}

// dE_tok[id,:] += sum over the tokens u with ids[u] = id of g[u,:], in ascending u.  One workgroup per
// token; the workgroup of the first occurrence of an id does the whole sum, the others leave at once.
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_tok_kernel(int Tn, int H, int V, const int* __restrict__ ids,
                                                            const T* __restrict__ g, float* __restrict__ dEtok) {
  __shared__ unsigned long long mask[4];
  const int t = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int id = clamp_id(ids[t], V);
  int earlier = 0;
  for (int u = tid; u < t; u += 256) earlier |= clamp_id(ids[u], V) == id;
  if (__syncthreads_or(earlier)) return;
  for (int c0 = 0; c0 < H; c0 += 256) {
    const int c = c0 + tid;
    float acc = 0.f;
    for (int base = (t / 256) * 256; base < Tn; base += 256) {
      const int u = base + tid;
      const bool hit = u >= t && u < Tn && clamp_id(ids[u], V) == id;
      const unsigned long long b = __ballot(hit);
      if (lane == 0) mask[wave] = b;
      __syncthreads();
      for (int w = 0; w < 4; ++w) {
        unsigned long long m = mask[w];
        while (m) {
          const int u2 = base + w * 64 + __ffsll((long long)m) - 1;
          m &= m - 1;
          if (c < H) acc += to_f32<T>(g[(long)u2 * H + c]);
        }
      }
      __syncthreads();
    }
    if (c < H) dEtok[(long)id * H + c] += acc;
  }
}

// dE_pos[p,:] += sum over the samples b of g[b*S + p,:], in ascending b
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_pos_kernel(int Tn, int S, int H, const T* __restrict__ g,
                                                            float* __restrict__ dEpos) {
  const int p = blockIdx.x, c = blockIdx.y * 256 + threadIdx.x;
  if (c >= H) return;
  float acc = 0.f;
  for (int u = p; u < Tn; u += S) acc += to_f32<T>(g[(long)u * H + c]);
  dEpos[(long)p * H + c] += acc;
}

__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  v = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  return v;
}
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  v = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  return v;
}

// per token: lse = log sum_v exp(logits[t,v]), loss_tok = lse - logits[t,label]; one workgroup per token
template <typename T>
__global__ __launch_bounds__(256) void xent_fwd_kernel(int V, const T* __restrict__ logits, const int* __restrict__ labels,
                                                       float* __restrict__ lse, float* __restrict__ loss_tok) {
  typedef typename V8<T>::type vec;
  __shared__ float red[4];
  const long t = blockIdx.x;
  const T* row = logits + t * V;
  float m = -INFINITY;
  for (int v = threadIdx.x * 8; v < V; v += 2048) {
    const vec x = *(const vec*)(row + v);
#pragma unroll
    for (int j = 0; j < 8; ++j) m = fmaxf(m, to_f32<T>(x[j]));
  }
  m = block_max(m, red);
  float s = 0.f;
  for (int v = threadIdx.x * 8; v < V; v += 2048) {
    const vec x = *(const vec*)(row + v);
#pragma unroll
    for (int j = 0; j < 8; ++j) s += expf(to_f32<T>(x[j]) - m);
  }
  s = block_sum(s, red);
  if (threadIdx.x == 0) {
    const float l = m + logf(s);
    lse[t] = l;
    loss_tok[t] = l - to_f32<T>(row[clamp_id(labels[t], V)]);
  }
}

// dlogits[t,v] = (exp(logits[t,v] - lse[t]) - [v = label]) * scale; may run in place
template <typename T>
__global__ __launch_bounds__(256) void xent_bwd_kernel(int V, const T* logits, const int* __restrict__ labels,
                                                       const float* __restrict__ lse, float scale, T* dlogits) {
  typedef typename V8<T>::type vec;
  const long t = blockIdx.x;
  const T* row = logits + t * V;
  T* out = dlogits + t * V;
  const float l = lse[t];
  const int lab = clamp_id(labels[t], V);
  for (int v = threadIdx.x * 8; v < V; v += 2048) {
    const vec x = *(const vec*)(row + v);
    vec o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = from_f32<T>((expf(to_f32<T>(x[j]) - l) - (v + j == lab ? 1.f : 0.f)) * scale);
    *(vec*)(out + v) = o;
  }
}

// out[0] = scale * sum_i in[i]: fixed order (strided partial sums per thread, then a fixed tree)
__global__ __launch_bounds__(256) void ordered_sum_kernel(long n, const float* __restrict__ in, float scale,
                                                          float* __restrict__ out) {
  __shared__ float red[256];
  float acc = 0.f;
  for (long i = threadIdx.x; i < n; i += 256) acc += in[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = red[0] * scale;
}

}  // namespace

hipError_t launch_embed_fwd(hipStream_t s, int dtype, int T, int S, int H, int V, const int* ids, const void* Etok,
                            const void* Epos, void* out) {
  if (T <= 0) return hipSuccess;
  const dim3 grid((T + 3) / 4), block(256);
  if (dtype == 1)
    hipLaunchKernelGGL(embed_fwd_kernel<bf16_t>, grid, block, 0, s, T, S, H, V, ids, (const bf16_t*)Etok,
                       (const bf16_t*)Epos, (bf16_t*)out);
  else
    hipLaunchKernelGGL(embed_fwd_kernel<float>, grid, block, 0, s, T, S, H, V, ids, (const float*)Etok,
                       (const float*)Epos, (float*)out);
  return hipGetLastError();
}

hipError_t launch_embed_bwd(hipStream_t s, int dtype, int T, int S, int H, int V, const int* ids, const void* g,
                            float* dEtok, float* dEpos) {
  if (T <= 0) return hipSuccess;
  const dim3 gp(S < T ? S : T, (H + 255) / 256);
  if (dtype == 1) {
    hipLaunchKernelGGL(embed_bwd_tok_kernel<bf16_t>, dim3(T), dim3(256), 0, s, T, H, V, ids, (const bf16_t*)g, dEtok);
    hipLaunchKernelGGL(embed_bwd_pos_kernel<bf16_t>, gp, dim3(256), 0, s, T, S, H, (const bf16_t*)g, dEpos);
  } else {
    hipLaunchKernelGGL(embed_bwd_tok_kernel<float>, dim3(T), dim3(256), 0, s, T, H, V, ids, (const float*)g, dEtok);
    hipLaunchKernelGGL(embed_bwd_pos_kernel<float>, gp, dim3(256), 0, s, T, S, H, (const float*)g, dEpos);
  }
  return hipGetLastError();
}

hipError_t launch_xent_fwd(hipStream_t s, int dtype, int T, int V, const void* logits, const int* labels, float* lse,
                           float* loss_tok) {
  if (T <= 0) return hipSuccess;
  if (dtype == 1)
    hipLaunchKernelGGL(xent_fwd_kernel<bf16_t>, dim3(T), dim3(256), 0, s, V, (const bf16_t*)logits, labels, lse, loss_tok);
  else
    hipLaunchKernelGGL(xent_fwd_kernel<float>, dim3(T), dim3(256), 0, s, V, (const float*)logits, labels, lse, loss_tok);
  return hipGetLastError();
}

hipError_t launch_xent_bwd(hipStream_t s, int dtype, int T, int V, const void* logits, const int* labels,
                           const float* lse, float scale, void* dlogits) {
  if (T <= 0) return hipSuccess;
  if (dtype == 1)
    hipLaunchKernelGGL(xent_bwd_kernel<bf16_t>, dim3(T), dim3(256), 0, s, V, (const bf16_t*)logits, labels, lse, scale,
                       (bf16_t*)dlogits);
  else
    hipLaunchKernelGGL(xent_bwd_kernel<float>, dim3(T), dim3(256), 0, s, V, (const float*)logits, labels, lse, scale,
                       (float*)dlogits);
  return hipGetLastError();
}

hipError_t launch_ordered_sum(hipStream_t s, long n, const float* in, float scale, float* out) {
  hipLaunchKernelGGL(ordered_sum_kernel, dim3(1), dim3(256), 0, s, n, in, scale, out);
  return hipGetLastError();
}

}  // namespace bamboo
