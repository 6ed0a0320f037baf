// Ordered final sum of partial rows, shared by the stand-alone reduction kernel and by the tail
// workgroups of the grouped weight-gradient launch.  The order of the additions is the same for any
// workgroup size: the rows are cut into kReduceGroups contiguous groups, each summed front to back, and
// the group sums are added in ascending order -- so both callers give the same bits.
#pragma once
#include "common.h"

namespace bamboo {

constexpr int kReduceGroups = 16;
constexpr int kReduceLdsFloats = 2 * kReduceGroups * 64;

// Workgroup `blk` of the batch: 64 columns of the segment whose block range holds blk.  red: LDS,
// kReduceLdsFloats floats.  blockDim.x must be a multiple of 64 that divides 64 * kReduceGroups.
// Must be reached by the whole workgroup.
__device__ __forceinline__ void colreduce_batch_block(const GradReduceBatch& batch, int blk, float* red) {
  int si = 0;
#pragma unroll
  for (int k = 1; k < 8; ++k)
    if (k < batch.n && blk >= batch.seg[k].block0) si = k;
  const GradReduceSeg sg = batch.seg[si];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int c = (blk - sg.block0) * 64 + lane;
  const int per = (sg.parts + kReduceGroups - 1) / kReduceGroups;
  const bool two = sg.p1 != nullptr;
  if (nw == kReduceGroups) {                       // one group per wavefront
    float s = 0.f, q = 0.f;
    if (c < sg.N) {
      const int y_end = min(sg.parts, (w + 1) * per);
#pragma unroll 8
      for (int y = w * per; y < y_end; ++y) s += sg.p0[(long)y * sg.N + c];
      if (two) {
#pragma unroll 8
        for (int y = w * per; y < y_end; ++y) q += sg.p1[(long)y * sg.N + c];
      }
    }
    red[w * 64 + lane] = s;
    red[(kReduceGroups + w) * 64 + lane] = q;
  } else {                                         // a wavefront walks its groups side by side (loads of all in flight)
    const int gpw = kReduceGroups / nw;            // groups w*gpw .. w*gpw + gpw - 1
    for (int g0 = w * gpw; g0 < (w + 1) * gpw; g0 += 4) {
      float s[4] = {0.f, 0.f, 0.f, 0.f}, q[4] = {0.f, 0.f, 0.f, 0.f};
      if (c < sg.N) {
        for (int y = 0; y < per; ++y) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int row = (g0 + j) * per + y;
            if (g0 + j < (w + 1) * gpw && row < sg.parts) {
              s[j] += sg.p0[(long)row * sg.N + c];
              if (two) q[j] += sg.p1[(long)row * sg.N + c];
            }
          }
        }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (g0 + j < (w + 1) * gpw) {
          red[(g0 + j) * 64 + lane] = s[j];
          red[(kReduceGroups + g0 + j) * 64 + lane] = q[j];
        }
    }
  }
  __syncthreads();
  if (w == 0 && c < sg.N) {
    float a = 0.f, b = 0.f;
#pragma unroll
    for (int k = 0; k < kReduceGroups; ++k) {
      a += red[k * 64 + lane];
      b += red[(kReduceGroups + k) * 64 + lane];
    }
    sg.out0[c] += a;
    if (two) sg.out1[c] += b;
  }
}

}  // namespace bamboo
