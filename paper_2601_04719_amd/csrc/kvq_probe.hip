// No-math streaming probes: what the memory system of this GPU sustains for the four traffic
// patterns of the library.  Read-only and write-only use a flat one-shot kernel with 16-byte
// wave-contiguous accesses: 16 KiB per workgroup for reads, and 4 KiB (one plain store per lane) for
// writes, which is what a pure write stream likes best here (6.8 TB/s; 6.0 with two or more stores
// per lane, 5.9 with nontemporal stores, 5.0 for a grid-stride loop).  The two mixed patterns run the production
// quantize / dequantize kernels with their arithmetic compiled out, i.e. exactly their loads,
// stores and launch shape.  Measurement aid only: what the probes write is meaningless as data.
#include "kvq_internal.h"

namespace kvq {

// mode 0: read fp32 (max-reduce to keep the loads live); mode 1: write fp32.  16 B per lane-access.
template <int MODE, int U>
__global__ __launch_bounds__(kBlock) void probe_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst,
                                                       int64_t nvec, float* __restrict__ sink) {
  const int64_t base = ((int64_t)blockIdx.x * U) * kBlock + threadIdx.x;
  f32x4 v[U];
  float acc = 0.0f;
#pragma unroll
  for (int u = 0; u < U; u++) {
    const int64_t i = base + (int64_t)u * kBlock;
    if (i < nvec) {
      if constexpr (MODE == 0) v[u] = __builtin_nontemporal_load(src + i);
    }
  }
#pragma unroll
  for (int u = 0; u < U; u++) {
    const int64_t i = base + (int64_t)u * kBlock;
    if (i < nvec) {
      if constexpr (MODE == 0) acc = fmaxf(acc, fmaxf(fmaxf(v[u].x, v[u].y), fmaxf(v[u].z, v[u].w)));
      if constexpr (MODE == 1) dst[i] = f32x4{1.0f, 2.0f, 3.0f, (float)i};
    }
  }
  if (MODE == 0 && acc == 12345.678f) *sink = acc;  // never true for the probe's inputs; keeps the loads
}

}  // namespace kvq

using namespace kvq;

extern "C" kvq_status kvq_probe_stream(int mode, const float* src_f32, float* dst_f32, const int8_t* src_i8,
                                       int8_t* dst_i8, const float* scales, int64_t batch, int64_t N, int64_t D,
                                       kvq_stream_t stream) {
  if (batch < 1 || N < 1 || D < 1 || D % 4) return KVQ_ERR_SHAPE;
  if (mode < 0 || mode > 3) return KVQ_ERR_ARG;
  if (((mode == 0 || mode == 2) && !src_f32) || ((mode == 1 || mode == 3) && !dst_f32) || (mode == 2 && !dst_i8) ||
      (mode == 3 && !src_i8) || (mode >= 2 && !scales))
    return KVQ_ERR_NULL;
  if (!aligned(src_f32, 16) || !aligned(dst_f32, 16) || !aligned(src_i8, 4) || !aligned(dst_i8, 4)) return KVQ_ERR_ARG;
  if (N > (INT64_MAX / 8) / D || batch > (INT64_MAX / 8) / (N * D)) return KVQ_ERR_OVERFLOW;
  if (mode >= 2) return launch_probe_codec(mode, src_f32, dst_f32, src_i8, dst_i8, scales, batch, N, D, stream);
  const int64_t nvec = batch * N * D / 4;
  constexpr int U = 4;
  const int64_t per_block = mode == 0 ? (int64_t)kBlock * U : kBlock;
  const int64_t blocks = (nvec + per_block - 1) / per_block;
  if (blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  const dim3 grid((uint32_t)blocks), block(kBlock);
  const f32x4* s = reinterpret_cast<const f32x4*>(src_f32);
  f32x4* d = reinterpret_cast<f32x4*>(dst_f32);
  // mode 0 needs a place for its never-taken store; any valid fp32 address will do
  float* sink = dst_f32 ? dst_f32 : const_cast<float*>(src_f32);
  if (mode == 0) hipLaunchKernelGGL((probe_kernel<0, U>), grid, block, 0, stream, s, d, nvec, sink);
  else hipLaunchKernelGGL((probe_kernel<1, 1>), grid, block, 0, stream, s, d, nvec, sink);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}
