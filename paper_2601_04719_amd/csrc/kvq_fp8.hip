// FP8 codes: the quantize / dequantize pair with an OCP E4M3 number as the 8-bit code
// (paper: Future Work, "GPU-specific numeric formats such as FP8"; the operations are
//  Eq. (quantize) / Eq. (dequantize) with the rounding to an integer in [-127, 127] replaced by
//  rounding to the nearest E4M3 value, ties to even, saturating at +-448; scale = absmax / 448).
//
// E4M3: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits; exponent field 0 is subnormal
// (multiples of 2^-9); the largest finite value is 448 (0x7E); 0x7F / 0xFF are NaN and never produced.
// The vector kernel encodes with the GPU's conversion instruction (v_cvt_pk_fp8_f32, OCP E4M3 on
// gfx950) after an explicit clamp to +-448, so that only its round-to-nearest-even inside the finite
// range is relied on; the scalar kernel (rows that cannot be moved as vectors) and the decoder work on
// the bit patterns, which spells the rounding out.  Both forms are checked bit for bit against the CPU
// oracle on a dense grid of quotients (every 4096th fp32 pattern, +-3 ulp around every rounding
// boundary, subnormals, the saturation edge).  On the bit patterns:
//  - encode: in the normal range the 23-bit fp32 mantissa is rounded to 3 bits by adding
//    0x7FFFF + (lowest kept bit) and shifting (a carry runs into the exponent, as it should), and the
//    exponent is rebiased by 127 - 7; below 2^-6, |y| * 2^9 is rounded to an integer 0..8 by adding
//    2^23; 448 and above saturates.
//  - decode: the 7 magnitude bits placed at bit 20 of an fp32 pattern are (1 + M/8) * 2^(E-127), or the
//    fp32 subnormal M * 2^-129 for E = 0; multiplying by 2^120 gives the E4M3 value exactly in both
//    cases (fp32 subnormals are not flushed in this library).
// Same streaming shape as the int8 kernels: a lane owns 4 adjacent channels.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

namespace {

// E4M3 bit pattern (low byte) of x / s; `keep` is 0 for a zero scale (code 0) and 0xff otherwise.
__device__ __forceinline__ uint32_t e4m3_of(float x, float s, uint32_t keep) {
  const float y = x / s;  // correctly rounded IEEE divide
  const uint32_t u = __float_as_uint(y);
  const uint32_t a = u & 0x7fffffffu;
  const uint32_t r = ((a + 0x7ffffu + ((a >> 20) & 1u)) >> 20) - 960u;
  const uint32_t q = __float_as_uint(__uint_as_float(a) * 512.0f + 8388608.0f) & 15u;
  uint32_t c = a < 0x3c800000u ? q : r;  // 0x3c800000 = 2^-6
  c = a >= 0x43e00000u ? 0x7eu : c;      // 0x43e00000 = 448
  return (c | ((u >> 24) & 0x80u)) & keep;
}

// value of E4M3 byte b of `word`, times the channel's scale (the first product is exact)
__device__ __forceinline__ float dq8(uint32_t word, int b, float s) {
  const uint32_t c = (word >> (8 * b)) & 0xffu;
  const float v = __uint_as_float(((c & 0x7fu) << 20) | ((c & 0x80u) << 24)) * __uint_as_float(0x7b800000u);  // 2^120
  return v * s;
}

template <int V, int U, bool NT>
__global__ __launch_bounds__(kMaxBlock) void quantize_fp8_kernel(const float* __restrict__ x,
                                                                 const float* __restrict__ scales,
                                                                 uint8_t* __restrict__ codes, int64_t N, int64_t D,
                                                                 int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                                 int64_t rows_per_chunk, int64_t groups) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * V;
  float ls[V];
  uint32_t keep[V];
#pragma unroll
  for (int i = 0; i < V; i++) {
    const float s = scales[it.slab * D + col + i];
    ls[i] = divisor_of(s);
    keep[i] = s == 0.0f ? 0u : 0xffu;
  }
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  const float* px = x + (it.slab * N + row) * D + col;
  uint8_t* pc = codes + (it.slab * N + row) * D + col;
  uint32_t kmask = 0;  // byte mask: 0x00 for channels with a zero scale
#pragma unroll
  for (int i = 0; i < V; i++) kmask |= keep[i] << (8 * i);
  if constexpr (V == 4) {
    auto do_rows = [&](auto nrows_tag) {
      constexpr int R = decltype(nrows_tag)::value;
      f32x4 v[R];
#pragma unroll
      for (int u = 0; u < R; u++) v[u] = ld<NT>(reinterpret_cast<const f32x4*>(px + u * step));
#pragma unroll
      for (int u = 0; u < R; u++) {
        // hardware conversion (v_cvt_pk_fp8_f32: OCP E4M3 on this GPU, round to nearest even) after an
        // explicit clamp to +-448, so that its behaviour outside the finite range never matters
        const float y0 = __builtin_amdgcn_fmed3f(v[u].x / ls[0], -448.0f, 448.0f);
        const float y1 = __builtin_amdgcn_fmed3f(v[u].y / ls[1], -448.0f, 448.0f);
        const float y2 = __builtin_amdgcn_fmed3f(v[u].z / ls[2], -448.0f, 448.0f);
        const float y3 = __builtin_amdgcn_fmed3f(v[u].w / ls[3], -448.0f, 448.0f);
        uint32_t w = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(y0, y1, 0, false);
        w = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(y2, y3, (int)w, true);
        w &= kmask;
        st<NT>(reinterpret_cast<uint32_t*>(pc + u * step), w);
      }
    };
    for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * step)
      do_rows(std::integral_constant<int, U>{});
    for (; row < it.row1; row += it.TY, px += step, pc += step) do_rows(std::integral_constant<int, 1>{});
  } else {
    for (; row < it.row1; row += it.TY, px += step, pc += step) *pc = (uint8_t)e4m3_of(*px, ls[0], keep[0]);
  }
}

template <int V, int U, bool NT>
__global__ __launch_bounds__(kMaxBlock) void dequantize_fp8_kernel(const uint8_t* __restrict__ codes,
                                                                   const float* __restrict__ scales,
                                                                   float* __restrict__ x_hat, int64_t N, int64_t D,
                                                                   int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                                   int64_t rows_per_chunk, int64_t groups) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * V;
  float s[V];
#pragma unroll
  for (int i = 0; i < V; i++) s[i] = scales[it.slab * D + col + i];
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  const uint8_t* pc = codes + (it.slab * N + row) * D + col;
  float* px = x_hat + (it.slab * N + row) * D + col;
  if constexpr (V == 4) {
    auto do_rows = [&](auto nrows_tag) {
      constexpr int R = decltype(nrows_tag)::value;
      uint32_t w[R];
#pragma unroll
      // codes without the streaming hint, as in dequantize_kernel: they may stay in the memory-side cache
      for (int u = 0; u < R; u++) w[u] = ld<false>(reinterpret_cast<const uint32_t*>(pc + u * step));
#pragma unroll
      for (int u = 0; u < R; u++) {
        const f32x4 o = {dq8(w[u], 0, s[0]), dq8(w[u], 1, s[1]), dq8(w[u], 2, s[2]), dq8(w[u], 3, s[3])};
        st<NT>(reinterpret_cast<f32x4*>(px + u * step), o);
      }
    };
    for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * step)
      do_rows(std::integral_constant<int, U>{});
    for (; row < it.row1; row += it.TY, px += step, pc += step) do_rows(std::integral_constant<int, 1>{});
  } else {
    for (; row < it.row1; row += it.TY, px += step, pc += step) *px = dq8(*pc, 0, s[0]);
  }
}

kvq_status fp8_tiling(int64_t batch, int64_t N, int64_t D, const void* fp32_ptr, const void* codes,
                      const float* scales, int default_unroll, int default_block, int* U_out, Tiling* t_out) {
  const bool wide = D % 4 == 0 && aligned(fp32_ptr, 16) && aligned(codes, 4) && aligned(scales, 16);
  return stream_tiling(batch, N, D, wide ? 4 : 1, wide, default_unroll, default_block, U_out, t_out);
}

#define KVQ_LAUNCH8(KERNEL, ...)                                                                               \
  do {                                                                                                         \
    const dim3 grid((uint32_t)t.items), block(t.block);                                                        \
    if (t.V == 1)                                                                                              \
      hipLaunchKernelGGL((KERNEL<1, 1, false>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2, t.ctiles, \
                         t.rchunks, t.rows_per_chunk, t.groups);                                               \
    else if (U == 1)                                                                                           \
      hipLaunchKernelGGL((KERNEL<4, 1, true>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2, t.ctiles,  \
                         t.rchunks, t.rows_per_chunk, t.groups);                                               \
    else if (U == 2)                                                                                           \
      hipLaunchKernelGGL((KERNEL<4, 2, true>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2, t.ctiles,  \
                         t.rchunks, t.rows_per_chunk, t.groups);                                               \
    else if (U == 4)                                                                                           \
      hipLaunchKernelGGL((KERNEL<4, 4, true>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2, t.ctiles,  \
                         t.rchunks, t.rows_per_chunk, t.groups);                                               \
    else                                                                                                       \
      hipLaunchKernelGGL((KERNEL<4, 8, true>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2, t.ctiles,  \
                         t.rchunks, t.rows_per_chunk, t.groups);                                               \
  } while (0)

}  // namespace

kvq_status launch_quantize_fp8(const float* x, const float* scales, uint8_t* codes, int64_t batch, int64_t N,
                               int64_t D, hipStream_t stream) {
  int U;
  Tiling t;
  if (kvq_status s = fp8_tiling(batch, N, D, x, codes, scales, 4, 512, &U, &t)) return s;
  KVQ_LAUNCH8(quantize_fp8_kernel, x, scales, codes);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

kvq_status launch_dequantize_fp8(const uint8_t* codes, const float* scales, float* x_hat, int64_t batch, int64_t N,
                                 int64_t D, hipStream_t stream) {
  int U;
  Tiling t;
  if (kvq_status s = fp8_tiling(batch, N, D, x_hat, codes, scales, 2, 256, &U, &t)) return s;
  KVQ_LAUNCH8(dequantize_fp8_kernel, codes, scales, x_hat);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
