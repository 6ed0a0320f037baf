// Adam update of a flat parameter vector and the helpers of the replica weight
// synchronisation.  HBM-bound: 16 bytes read and 12 + sizeof(storage) bytes
// written per parameter, 16-byte accesses, no reductions.
//
// The paper names the optimizer (Adam, Section 7) and requires the replica to
// carry the successor's parameters and optimizer state (Section 5.1); the update
// is the textbook one: m <- b1 m + (1-b1) g, v <- b2 v + (1-b2) g^2,
// w <- w - lr (m / (1-b1^t)) / (sqrt(v / (1-b2^t)) + eps), on fp32 master
// weights, with the storage-dtype copy that the layer kernels read rewritten in
// the same pass.
#include <math.h>

#include "common.h"

namespace bamboo {

template <typename T> struct Store4;
template <> struct Store4<float> {
  __device__ static __forceinline__ void put(float* p, const float4& v) { *(float4*)p = v; }
  __device__ static __forceinline__ float4 get(const float* p) { return *(const float4*)p; }
};
template <> struct Store4<bf16_t> {
  typedef __attribute__((ext_vector_type(4))) __bf16 raw;
  __device__ static __forceinline__ void put(bf16_t* p, const float4& v) {
    raw t;
    t[0] = (bf16_t)v.x; t[1] = (bf16_t)v.y; t[2] = (bf16_t)v.z; t[3] = (bf16_t)v.w;
    *(raw*)p = t;
  }
  __device__ static __forceinline__ float4 get(const bf16_t* p) {
    const raw t = *(const raw*)p;
    return make_float4((float)t[0], (float)t[1], (float)t[2], (float)t[3]);
  }
};

// inv_c1 = 1 / (1 - beta1^t), inv_c2 = 1 / (1 - beta2^t), computed on the host in double
template <typename T>
__global__ __launch_bounds__(256) void adam_kernel(long n4, const float* __restrict__ g, float* __restrict__ master,
                                                   float* __restrict__ m, float* __restrict__ v, T* __restrict__ w,
                                                   float lr, float beta1, float beta2, float eps, float inv_c1,
                                                   float inv_c2) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n4; i += (long)gridDim.x * 256) {
    const float4 gg = ((const float4*)g)[i];
    float4 mm = ((const float4*)m)[i], vv = ((const float4*)v)[i], ww = ((const float4*)master)[i];
    const float gs[4] = {gg.x, gg.y, gg.z, gg.w};
    float ms[4] = {mm.x, mm.y, mm.z, mm.w}, vs[4] = {vv.x, vv.y, vv.z, vv.w}, ws[4] = {ww.x, ww.y, ww.z, ww.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      ms[j] = beta1 * ms[j] + (1.0f - beta1) * gs[j];
      vs[j] = beta2 * vs[j] + (1.0f - beta2) * gs[j] * gs[j];
      ws[j] -= lr * (ms[j] * inv_c1) / (sqrtf(vs[j] * inv_c2) + eps);
    }
    ((float4*)m)[i] = make_float4(ms[0], ms[1], ms[2], ms[3]);
    ((float4*)v)[i] = make_float4(vs[0], vs[1], vs[2], vs[3]);
    const float4 wo = make_float4(ws[0], ws[1], ws[2], ws[3]);
    ((float4*)master)[i] = wo;
    Store4<T>::put(w + 4 * i, wo);
  }
}

// master[i] = (float) w[i]
template <typename T>
__global__ __launch_bounds__(256) void widen_kernel(long n4, const T* __restrict__ w, float* __restrict__ master) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n4; i += (long)gridDim.x * 256)
    ((float4*)master)[i] = Store4<T>::get(w + 4 * i);
}

__global__ __launch_bounds__(256) void fill_zero_kernel(long n4, float* __restrict__ p) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n4; i += (long)gridDim.x * 256)
    ((float4*)p)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

static unsigned grid_for(long n4) {
  long blocks = (n4 + 255) / 256;
  if (blocks > 256 * 8) blocks = 256 * 8;
  if (blocks < 1) blocks = 1;
  return (unsigned)blocks;
}

hipError_t launch_adam(hipStream_t s, int dtype, long n, const float* g, float* master, float* m, float* v, void* w,
                       float lr, float beta1, float beta2, float eps, int step) {
  if (n % 4 || step < 1) return hipErrorInvalidValue;
  const float inv_c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
  const float inv_c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
  const long n4 = n / 4;
  if (dtype == 0)
    hipLaunchKernelGGL(adam_kernel<float>, dim3(grid_for(n4)), dim3(256), 0, s, n4, g, master, m, v, (float*)w, lr, beta1,
                       beta2, eps, inv_c1, inv_c2);
  else
    hipLaunchKernelGGL(adam_kernel<bf16_t>, dim3(grid_for(n4)), dim3(256), 0, s, n4, g, master, m, v, (bf16_t*)w, lr,
                       beta1, beta2, eps, inv_c1, inv_c2);
  return hipGetLastError();
}

hipError_t launch_widen(hipStream_t s, int dtype, long n, const void* w, float* master) {
  if (n % 4) return hipErrorInvalidValue;
  const long n4 = n / 4;
  if (dtype == 0)
    hipLaunchKernelGGL(widen_kernel<float>, dim3(grid_for(n4)), dim3(256), 0, s, n4, (const float*)w, master);
  else
    hipLaunchKernelGGL(widen_kernel<bf16_t>, dim3(grid_for(n4)), dim3(256), 0, s, n4, (const bf16_t*)w, master);
  return hipGetLastError();
}

hipError_t launch_fill_zero(hipStream_t s, long n, float* p) {
  if (n % 4) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(n / 4)), dim3(256), 0, s, n / 4, p);
  return hipGetLastError();
}

}  // namespace bamboo
