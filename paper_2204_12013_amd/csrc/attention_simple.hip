// Softmax attention forward/backward on the vector ALUs (fp32 arithmetic, any
// sequence length, head size up to 128).  Used by the fp32 configuration and as
// the fallback of the bf16 path.  Online softmax over key tiles; the forward
// keeps only the per-row log-sum-exp, the backward recomputes the
// probabilities from it.  No atomics: dQ and dK/dV come from two kernels that
// each own their output rows, so results are bitwise reproducible.
#include "common.h"

namespace bamboo {

constexpr int QT = 16;  // rows owned by a block
constexpr int KT = 32;  // rows streamed per tile

template <typename T>
__device__ __forceinline__ void load_tile(float* dst, int ld, const T* src, long row_stride, int row0, int nrows,
                                          int row_limit, int D) {
  // dst[r][c] = src[(row0 + r) * row_stride + c] for r < nrows, zero beyond row_limit
  for (int idx = threadIdx.x; idx < nrows * D; idx += blockDim.x) {
    const int r = idx / D, c = idx % D;
    float v = 0.f;
    if (row0 + r < row_limit) v = to_f32<T>(src[(long)(row0 + r) * row_stride + c]);
    dst[r * ld + c] = v;
  }
}

__device__ __forceinline__ float group16_max(float v) {
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float group16_sum(float v) {
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_simple_kernel(AttnDesc a) {
  extern __shared__ float smem[];
  const int D = a.d, ld = D + 1, H = a.heads * D;
  float* Qs = smem;
  float* Ks = Qs + QT * ld;
  float* Vs = Ks + KT * ld;
  float* Ps = Vs + KT * ld;  // [QT][KT+1]
  const int b = blockIdx.y / a.heads, h = blockIdx.y % a.heads;
  const int q0 = blockIdx.x * QT;
  const int q = threadIdx.x / 16, t = threadIdx.x % 16;
  const T* base = (const T*)a.qkv + (long)b * a.S * 3 * H + h * D;
  const float scale = rsqrtf((float)D);
  load_tile<T>(Qs, ld, base, 3 * H, q0, QT, a.S, D);
  const int qrow = q0 + q;
  float m = -INFINITY, l = 0.f, o[8] = {};
  const int kend = a.causal ? min(a.S, q0 + QT) : a.S;
  for (int k0 = 0; k0 < kend; k0 += KT) {
    __syncthreads();
    load_tile<T>(Ks, ld, base + H, 3 * H, k0, KT, a.S, D);
    load_tile<T>(Vs, ld, base + 2 * H, 3 * H, k0, KT, a.S, D);
    __syncthreads();
    float sc[2];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const int j = t + 16 * jj, key = k0 + j;
      const bool valid = key < a.S && qrow < a.S && (!a.causal || key <= qrow);
      float dot = 0.f;
      for (int c = 0; c < D; ++c) dot = fmaf(Qs[q * ld + c], Ks[j * ld + c], dot);
      sc[jj] = valid ? dot * scale : -INFINITY;
    }
    const float mnew = fmaxf(m, group16_max(fmaxf(sc[0], sc[1])));
    const float corr = (m == -INFINITY) ? 0.f : __expf(m - mnew);
    float psum = 0.f;
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const float p = (sc[jj] == -INFINITY) ? 0.f : __expf(sc[jj] - mnew);
      Ps[q * (KT + 1) + t + 16 * jj] = p;
      psum += p;
    }
    l = l * corr + group16_sum(psum);
    m = mnew;
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = t + 16 * e;
      if (c < D) {
        float acc = o[e] * corr;
        for (int j = 0; j < KT; ++j) acc = fmaf(Ps[q * (KT + 1) + j], Vs[j * ld + c], acc);
        o[e] = acc;
      }
    }
  }
  if (qrow < a.S) {
    const float inv = 1.f / l;
    T* out = (T*)a.ctx + ((long)b * a.S + qrow) * H + h * D;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = t + 16 * e;
      if (c < D) out[c] = from_f32<T>(o[e] * inv);
    }
    if (t == 0) a.lse[((long)b * a.heads + h) * a.S + qrow] = m + __logf(l);
  }
}

// delta[b,h,i] = sum_c dctx[i,c] * ctx[i,c] over the head's columns
template <typename T>
__global__ void attn_delta_kernel(AttnDesc a) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long total = (long)a.B * a.heads * a.S;
  if (idx >= total) return;
  const int i = idx % a.S;
  const int h = (idx / a.S) % a.heads;
  const int b = idx / ((long)a.S * a.heads);
  const int H = a.heads * a.d;
  const long off = ((long)b * a.S + i) * H + h * a.d;
  const T* o = (const T*)a.ctx + off;
  const T* dO = (const T*)a.dctx + off;
  float s = 0.f;
  for (int c = 0; c < a.d; ++c) s = fmaf(to_f32<T>(o[c]), to_f32<T>(dO[c]), s);
  a.delta[idx] = s;
}

// dQ: a block owns QT query rows and streams the keys.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_simple_kernel(AttnDesc a) {
  extern __shared__ float smem[];
  const int D = a.d, ld = D + 1, H = a.heads * D;
  float* Qs = smem;
  float* dOs = Qs + QT * ld;
  float* Ks = dOs + QT * ld;
  float* Vs = Ks + KT * ld;
  float* dSs = Vs + KT * ld;  // [QT][KT+1]
  const int b = blockIdx.y / a.heads, h = blockIdx.y % a.heads;
  const int q0 = blockIdx.x * QT;
  const int q = threadIdx.x / 16, t = threadIdx.x % 16;
  const T* base = (const T*)a.qkv + (long)b * a.S * 3 * H + h * D;
  const T* dbase = (const T*)a.dctx + (long)b * a.S * H + h * D;
  const float scale = rsqrtf((float)D);
  load_tile<T>(Qs, ld, base, 3 * H, q0, QT, a.S, D);
  load_tile<T>(dOs, ld, dbase, H, q0, QT, a.S, D);
  const int qrow = q0 + q;
  const long sidx = ((long)b * a.heads + h) * a.S + qrow;
  const float lse = qrow < a.S ? a.lse[sidx] : 0.f;
  const float delta = qrow < a.S ? a.delta[sidx] : 0.f;
  float dq[8] = {};
  const int kend = a.causal ? min(a.S, q0 + QT) : a.S;
  for (int k0 = 0; k0 < kend; k0 += KT) {
    __syncthreads();
    load_tile<T>(Ks, ld, base + H, 3 * H, k0, KT, a.S, D);
    load_tile<T>(Vs, ld, base + 2 * H, 3 * H, k0, KT, a.S, D);
    __syncthreads();
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      const int j = t + 16 * jj, key = k0 + j;
      const bool valid = key < a.S && qrow < a.S && (!a.causal || key <= qrow);
      float dot = 0.f, dp = 0.f;
      for (int c = 0; c < D; ++c) {
        dot = fmaf(Qs[q * ld + c], Ks[j * ld + c], dot);
        dp = fmaf(dOs[q * ld + c], Vs[j * ld + c], dp);
      }
      const float p = valid ? __expf(dot * scale - lse) : 0.f;
      dSs[q * (KT + 1) + j] = p * (dp - delta);
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = t + 16 * e;
      if (c < D) {
        float acc = dq[e];
        for (int j = 0; j < KT; ++j) acc = fmaf(dSs[q * (KT + 1) + j], Ks[j * ld + c], acc);
        dq[e] = acc;
      }
    }
  }
  if (qrow < a.S) {
    T* out = (T*)a.dqkv + ((long)b * a.S + qrow) * 3 * H + h * D;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = t + 16 * e;
      if (c < D) out[c] = from_f32<T>(dq[e] * scale);
    }
  }
}

// dK, dV: a block owns QT key rows and streams the queries.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_simple_kernel(AttnDesc a) {
  extern __shared__ float smem[];
  const int D = a.d, ld = D + 1, H = a.heads * D;
  float* Ks = smem;
  float* Vs = Ks + QT * ld;
  float* Qs = Vs + QT * ld;
  float* dOs = Qs + KT * ld;
  float* Ps = dOs + KT * ld;      // [KT][QT+1]
  float* dSs = Ps + KT * (QT + 1);  // [KT][QT+1]
  const int b = blockIdx.y / a.heads, h = blockIdx.y % a.heads;
  const int k0 = blockIdx.x * QT;
  const int j = threadIdx.x / 16, t = threadIdx.x % 16;
  const T* base = (const T*)a.qkv + (long)b * a.S * 3 * H + h * D;
  const T* dbase = (const T*)a.dctx + (long)b * a.S * H + h * D;
  const float scale = rsqrtf((float)D);
  load_tile<T>(Ks, ld, base + H, 3 * H, k0, QT, a.S, D);
  load_tile<T>(Vs, ld, base + 2 * H, 3 * H, k0, QT, a.S, D);
  const int key = k0 + j;
  float dk[8] = {}, dv[8] = {};
  const int qbeg = a.causal ? (k0 / KT) * KT : 0;
  for (int q0 = qbeg; q0 < a.S; q0 += KT) {
    __syncthreads();
    load_tile<T>(Qs, ld, base, 3 * H, q0, KT, a.S, D);
    load_tile<T>(dOs, ld, dbase, H, q0, KT, a.S, D);
    __syncthreads();
#pragma unroll
    for (int ii = 0; ii < 2; ++ii) {
      const int i = t + 16 * ii, qrow = q0 + i;
      const bool valid = key < a.S && qrow < a.S && (!a.causal || key <= qrow);
      float dot = 0.f, dp = 0.f;
      for (int c = 0; c < D; ++c) {
        dot = fmaf(Qs[i * ld + c], Ks[j * ld + c], dot);
        dp = fmaf(dOs[i * ld + c], Vs[j * ld + c], dp);
      }
      float p = 0.f, ds = 0.f;
      if (valid) {
        const long sidx = ((long)b * a.heads + h) * a.S + qrow;
        p = __expf(dot * scale - a.lse[sidx]);
        ds = p * (dp - a.delta[sidx]);
      }
      Ps[i * (QT + 1) + j] = p;
      dSs[i * (QT + 1) + j] = ds;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = t + 16 * e;
      if (c < D) {
        float av = dv[e], ak = dk[e];
        for (int i = 0; i < KT; ++i) {
          av = fmaf(Ps[i * (QT + 1) + j], dOs[i * ld + c], av);
          ak = fmaf(dSs[i * (QT + 1) + j], Qs[i * ld + c], ak);
        }
        dv[e] = av;
        dk[e] = ak;
      }
    }
  }
  if (key < a.S) {
    T* out = (T*)a.dqkv + ((long)b * a.S + key) * 3 * H + h * D;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int c = t + 16 * e;
      if (c < D) {
        out[H + c] = from_f32<T>(dk[e] * scale);
        out[2 * H + c] = from_f32<T>(dv[e]);
      }
    }
  }
}

template <typename T>
static hipError_t fwd_impl(hipStream_t s, const AttnDesc& a) {
  const size_t sh = ((size_t)(QT + 2 * KT) * (a.d + 1) + QT * (KT + 1)) * sizeof(float);
  dim3 grid((a.S + QT - 1) / QT, a.B * a.heads);
  hipLaunchKernelGGL(attn_fwd_simple_kernel<T>, grid, dim3(256), sh, s, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t bwd_impl(hipStream_t s, const AttnDesc& a) {
  const long total = (long)a.B * a.heads * a.S;
  hipLaunchKernelGGL(attn_delta_kernel<T>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a);
  dim3 grid((a.S + QT - 1) / QT, a.B * a.heads);
  const size_t sh1 = ((size_t)(2 * QT + 2 * KT) * (a.d + 1) + QT * (KT + 1)) * sizeof(float);
  hipLaunchKernelGGL(attn_bwd_dq_simple_kernel<T>, grid, dim3(256), sh1, s, a);
  const size_t sh2 = ((size_t)(2 * QT + 2 * KT) * (a.d + 1) + 2 * KT * (QT + 1)) * sizeof(float);
  hipLaunchKernelGGL(attn_bwd_dkv_simple_kernel<T>, grid, dim3(256), sh2, s, a);
  return hipGetLastError();
}

hipError_t launch_attention_fwd_simple(hipStream_t s, int dtype, const AttnDesc& a) {
  if (a.d > 128) return hipErrorInvalidValue;
  return dtype == 0 ? fwd_impl<float>(s, a) : fwd_impl<bf16_t>(s, a);
}
hipError_t launch_attention_bwd_simple(hipStream_t s, int dtype, const AttnDesc& a) {
  if (a.d > 128) return hipErrorInvalidValue;
  return dtype == 0 ? bwd_impl<float>(s, a) : bwd_impl<bf16_t>(s, a);
}

hipError_t launch_attention_fwd(hipStream_t s, int dtype, const AttnDesc& a) {
  if (dtype == 1) {
    hipError_t e = launch_attention_fwd_mfma(s, a);
    if (e != hipErrorNotSupported) return e;
  }
  return launch_attention_fwd_simple(s, dtype, a);
}
hipError_t launch_attention_bwd(hipStream_t s, int dtype, const AttnDesc& a) {
  if (dtype == 1) {
    hipError_t e = launch_attention_bwd_mfma(s, a);
    if (e != hipErrorNotSupported) return e;
  }
  return launch_attention_bwd_simple(s, dtype, a);
}

}  // namespace bamboo
