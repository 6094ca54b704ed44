// No-math streaming probes: what the memory system of this GPU sustains for the four traffic
// patterns of the library.  Read-only and write-only use a flat one-shot kernel with 16-byte
// wave-contiguous accesses: 16 KiB per workgroup for reads, and 4 KiB (one plain store per lane) for
// writes, which is what a pure write stream likes best here (6.8 TB/s; 6.0 with two or more stores
// per lane, 5.9 with nontemporal stores, 5.0 for a grid-stride loop).  The two mixed patterns run the production
// quantize / dequantize kernels with their arithmetic compiled out, i.e. exactly their loads,
// stores and launch shape.  Measurement aid only: what the probes write is meaningless as data.
//
// This file also holds the other entry points of include/kvq_bench.h: the shader-clock probe, the
// paper's kernel designs as ablation points, the per-thread launch options and the host-side launch
// plan.  None of them is part of the method's interface.
#include <limits.h>

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

// One wavefront spins until the 100 MHz wall clock has advanced by `ticks10ns`, then reports how far the
// shader-clock counter moved meanwhile.  The loop ends on the wall clock, which always advances.
__global__ __launch_bounds__(64) void clock_probe_kernel(unsigned long long* __restrict__ out,
                                                         unsigned long long ticks10ns) {
  const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
  unsigned long long r1 = r0;
  while (r1 - r0 < ticks10ns) {
    __builtin_amdgcn_s_sleep(32);
    r1 = __builtin_amdgcn_s_memrealtime();
  }
  const unsigned long long c1 = __builtin_amdgcn_s_memtime();
  if (threadIdx.x == 0) {
    out[0] = c1 - c0;
    out[1] = r1 - r0;
  }
}

}  // namespace kvq

using namespace kvq;

extern "C" kvq_status kvq_probe_clock(uint64_t* ticks_out, int microseconds, kvq_stream_t stream) {
  if (!ticks_out) return KVQ_ERR_NULL;
  if (!aligned(ticks_out, 8) || microseconds < 1 || microseconds > 1000000) return KVQ_ERR_ARG;
  hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, stream,
                     reinterpret_cast<unsigned long long*>(ticks_out), (unsigned long long)microseconds * 100ull);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

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

extern "C" {

kvq_status kvq_quantize_variant(int variant, const float* x, const float* scales, int8_t* codes, int64_t batch,
                                int64_t N, int64_t D, kvq_stream_t stream) {
  if (!x || !scales || !codes) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (variant == KVQ_VARIANT_PRODUCTION) return launch_quantize(x, scales, codes, batch, N, D, stream);
  if (variant < KVQ_VARIANT_PRODUCTION || variant > KVQ_VARIANT_VECTORIZED) return KVQ_ERR_ARG;
  return launch_quantize_variant(variant, x, scales, codes, batch, N, D, stream);
}

kvq_status kvq_plan(int call, int64_t batch, int64_t N, int64_t D, int vector_access, int compute_units,
                    int64_t* plan_out) {
  if (!plan_out) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (compute_units < 1 || compute_units > 65536) return KVQ_ERR_ARG;
  int J = 1, U = 1;
  Tiling t;
  if (call == KVQ_PLAN_ABSMAX) {
    if (kvq_status s = absmax_plan(compute_units, batch, N, D, vector_access && D % 4 == 0, &J, &U, &t)) return s;
    t.V /= J;
  } else if (call == KVQ_PLAN_QUANTIZE || call == KVQ_PLAN_DEQUANTIZE) {
    const int V = vector_access ? pick_width(D, nullptr, nullptr, options().codec_width) : 1;
    const bool q = call == KVQ_PLAN_QUANTIZE;
    if (kvq_status s = stream_tiling_for(compute_units, batch, N, D, V, V > 1, q ? kQuantUnroll : kDequantUnroll,
                                         q ? kQuantBlock : dequant_block_for(D), &U, &t))
      return s;
  } else {
    return KVQ_ERR_ARG;
  }
  plan_out[0] = t.V;
  plan_out[1] = J;
  plan_out[2] = t.block;
  plan_out[3] = (int64_t)1 << t.tx_log2;
  plan_out[4] = t.ctiles;
  plan_out[5] = t.rchunks;
  plan_out[6] = t.rows_per_chunk;
  plan_out[7] = U;
  return KVQ_OK;
}

kvq_status kvq_set_option(int key, int value) {
  Options& o = options();
  switch (key) {
    case KVQ_OPT_CODEC_WIDTH:
      if (value != 4 && value != 8 && value != 16) return KVQ_ERR_ARG;
      o.codec_width = value;
      return KVQ_OK;
    case KVQ_OPT_CODEC_UNROLL:
      if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return KVQ_ERR_ARG;
      o.codec_unroll = value;
      return KVQ_OK;
    case KVQ_OPT_BLOCKS_PER_CU:
      if (value < 0 || value > 64) return KVQ_ERR_ARG;
      o.blocks_per_cu = value;
      return KVQ_OK;
    case KVQ_OPT_NONTEMPORAL:
      if (value != 0 && value != 1) return KVQ_ERR_ARG;
      o.nontemporal = value;
      return KVQ_OK;
    case KVQ_OPT_BLOCK_THREADS:
      if (value != 0 && value != 64 && value != 128 && value != 256 && value != 512) return KVQ_ERR_ARG;
      o.block_threads = value;
      return KVQ_OK;
    case KVQ_OPT_PASSES_PER_BLOCK:
      if (value < 0 || value > 65536) return KVQ_ERR_ARG;
      o.passes_per_block = value;
      return KVQ_OK;
    case KVQ_OPT_ABSMAX_UNROLL:
      if (value != 4 && value != 8 && value != 16) return KVQ_ERR_ARG;
      o.absmax_unroll = value;
      return KVQ_OK;
    case KVQ_OPT_ABSMAX_PASSES:
      if (value < 0 || value > 65536) return KVQ_ERR_ARG;
      o.absmax_passes = value;
      return KVQ_OK;
    case KVQ_OPT_ABSMAX_BLOCKS_PER_CU:
      if (value < 1 || value > 64) return KVQ_ERR_ARG;
      o.absmax_blocks_per_cu = value;
      return KVQ_OK;
    case KVQ_OPT_APPEND_BLOCKS_PER_CU:
      if (value < 1 || value > 1024) return KVQ_ERR_ARG;
      o.append_blocks_per_cu = value;
      return KVQ_OK;
    case KVQ_OPT_ABSMAX_SPAN:
      if (value != 1 && value != 2 && value != 4 && value != 8) return KVQ_ERR_ARG;
      o.absmax_span = value;
      return KVQ_OK;
    case KVQ_OPT_FUSED_MIN_LANES:
      if (value < 4 || value > 1024 || (value & (value - 1))) return KVQ_ERR_ARG;
      o.fused_min_lanes = value;
      return KVQ_OK;
    case KVQ_OPT_FUSED_MAX_ROWS:
      if (value != 0 && value != 4 && value != 8 && value != 16) return KVQ_ERR_ARG;
      o.fused_max_rows = value;
      return KVQ_OK;
    case KVQ_OPT_ATTN_FORM:
      if (value != 0 && value != 1) return KVQ_ERR_ARG;
      o.attn_form = value;
      return KVQ_OK;
    case KVQ_OPT_FUSED_TALL:
      if (value < 0 || value > 3) return KVQ_ERR_ARG;
      o.fused_tall = value;
      return KVQ_OK;
    default:
      return KVQ_ERR_ARG;
  }
}

int kvq_get_option(int key) {
  const Options& o = options();
  switch (key) {
    case KVQ_OPT_CODEC_WIDTH: return o.codec_width;
    case KVQ_OPT_CODEC_UNROLL: return o.codec_unroll;
    case KVQ_OPT_BLOCKS_PER_CU: return o.blocks_per_cu;
    case KVQ_OPT_NONTEMPORAL: return o.nontemporal;
    case KVQ_OPT_BLOCK_THREADS: return o.block_threads;
    case KVQ_OPT_PASSES_PER_BLOCK: return o.passes_per_block;
    case KVQ_OPT_ABSMAX_UNROLL: return o.absmax_unroll;
    case KVQ_OPT_ABSMAX_PASSES: return o.absmax_passes;
    case KVQ_OPT_ABSMAX_SPAN: return o.absmax_span;
    case KVQ_OPT_ABSMAX_BLOCKS_PER_CU: return o.absmax_blocks_per_cu;
    case KVQ_OPT_APPEND_BLOCKS_PER_CU: return o.append_blocks_per_cu;
    case KVQ_OPT_FUSED_MIN_LANES: return o.fused_min_lanes;
    case KVQ_OPT_FUSED_MAX_ROWS: return o.fused_max_rows;
    case KVQ_OPT_ATTN_FORM: return o.attn_form;
    case KVQ_OPT_FUSED_TALL: return o.fused_tall;
    default: return INT_MIN;
  }
}

}  // extern "C"
