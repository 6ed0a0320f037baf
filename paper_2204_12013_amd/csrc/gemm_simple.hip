// Generic strided GEMM on the vector ALUs with fp32 accumulation: the fp32
// configuration's GEMM and the fallback for bf16 shapes the MFMA kernel does
// not cover.  64x64 output tile, 16-deep k-slices staged in LDS, 4x4 outputs
// per thread; every access is bounds-checked so any M, N, K works.
#include "common.h"

namespace bamboo {

template <typename T>
__device__ __forceinline__ void epilogue_store(const GemmDesc& d, int m, int n, float acc) {
  const long i = (long)m * d.N + n;
  switch (d.epi) {
    case EPI_STORE:
      ((T*)d.C)[i] = from_f32<T>(acc);
      break;
    case EPI_BIAS:
      ((T*)d.C)[i] = from_f32<T>(acc + to_f32<T>(((const T*)d.bias)[n]));
      break;
    case EPI_BIAS_RES:
      ((T*)d.C)[i] = from_f32<T>(acc + to_f32<T>(((const T*)d.bias)[n]) + to_f32<T>(((const T*)d.res)[i]));
      break;
    case EPI_BIAS_GELU: {
      const float h = acc + to_f32<T>(((const T*)d.bias)[n]);
      ((T*)d.C)[i] = from_f32<T>(gelu_grad_f(h));
      ((T*)d.aux_out)[i] = from_f32<T>(gelu_f(h));
      break;
    }
    case EPI_RES:
      ((T*)d.C)[i] = from_f32<T>(acc + to_f32<T>(((const T*)d.res)[i]));
      break;
    case EPI_MUL:
      ((T*)d.C)[i] = from_f32<T>(acc * to_f32<T>(((const T*)d.aux_in)[i]));
      break;
    case EPI_ACC_F32:
      ((float*)d.C)[i] += acc;
      break;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void gemm_simple_kernel(GemmDesc d) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const T* A = (const T*)d.A;
  const T* B = (const T*)d.B;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < d.K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      int m, k;
      if (d.a_sk == 1) { k = idx % BK; m = idx / BK; } else { m = idx % BM; k = idx / BM; }
      float v = 0.f;
      if (m0 + m < d.M && k0 + k < d.K) v = to_f32<T>(A[(long)(m0 + m) * d.a_sm + (long)(k0 + k) * d.a_sk]);
      As[k][m] = v;
      int n, kb;
      if (d.b_sn == 1) { n = idx % BN; kb = idx / BN; } else { kb = idx % BK; n = idx / BK; }
      float w = 0.f;
      if (n0 + n < d.N && k0 + kb < d.K) w = to_f32<T>(B[(long)(k0 + kb) * d.b_sk + (long)(n0 + n) * d.b_sn]);
      Bs[kb][n] = w;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < d.M && n < d.N) epilogue_store<T>(d, m, n, acc[i][j]);
    }
}

hipError_t launch_gemm_simple(hipStream_t s, int dtype, const GemmDesc& d) {
  if (d.M <= 0 || d.N <= 0) return hipSuccess;
  dim3 grid((d.N + 63) / 64, (d.M + 63) / 64);
  if (dtype == 0)
    hipLaunchKernelGGL(gemm_simple_kernel<float>, grid, dim3(256), 0, s, d);
  else
    hipLaunchKernelGGL(gemm_simple_kernel<bf16_t>, grid, dim3(256), 0, s, d);
  return hipGetLastError();
}

hipError_t launch_gemm(hipStream_t s, int dtype, const GemmDesc& d) {
  if (d.colsum_out != nullptr) {   // bias gradient: dY is the B operand [K rows, N] of the weight-gradient form
    hipError_t e = launch_colsum_acc(s, dtype, d.K, d.N, d.B, d.colsum_out, d.colsum_partial);
    if (e != hipSuccess) return e;
  }
  if (dtype == 1) {
    hipError_t e = launch_gemm_mfma(s, d);
    if (e != hipErrorNotSupported) return e;
  }
  const hipError_t e = launch_gemm_simple(s, dtype, d);
  if (e != hipSuccess) return e;
  if (d.tile_colsum != nullptr && d.tile_colsum_parts != nullptr)   // the MFMA epilogue would have summed the columns
    return launch_colsum_partials(s, dtype, d.M, d.N, d.C, d.tile_colsum, d.tile_colsum_parts);
  return hipSuccess;
}

hipError_t launch_gemm_group(hipStream_t s, int dtype, const GemmDesc* d, int n, const GradReduceBatch* tail,
                             bool* tail_done) {
  if (tail_done) *tail_done = false;
  if (dtype == 1 && n > 1) {
    bool plain = true;
    for (int i = 0; i < n; ++i) plain = plain && d[i].colsum_out == nullptr;
    if (plain) {
      const hipError_t e = launch_gemm_group_mfma(s, d, n, tail_done ? tail : nullptr);
      if (e != hipErrorNotSupported) {
        if (tail_done) *tail_done = e == hipSuccess && tail != nullptr;
        return e;
      }
    }
  }
  for (int i = 0; i < n; ++i) {
    const hipError_t e = launch_gemm(s, dtype, d[i]);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace bamboo
