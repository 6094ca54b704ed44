// Workgroup-level reductions shared by the error-statistics kernels (device code only).
#pragma once

#include "kvq_internal.h"

namespace kvq {

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_down(v, off, 64));
  return v;
}

// Workgroup-wide (sum, max); the result is valid in thread 0.
__device__ __forceinline__ void block_reduce(double& sum, float& mx) {
  __shared__ double s_sum[kBlock / 64];
  __shared__ float s_max[kBlock / 64];
  sum = wave_sum(sum);
  mx = wave_max(mx);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
    s_sum[wave] = sum;
    s_max[wave] = mx;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kBlock / 64; w++) {
      sum += s_sum[w];
      mx = fmaxf(mx, s_max[w]);
    }
  }
}


}  // namespace kvq
