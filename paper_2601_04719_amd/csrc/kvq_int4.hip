// 4-bit codes: the quantize / dequantize pair with the integer range [-7, 7]
// (paper: Limitations, "Lower bit-widths"; the operations are Eq. (quantize) /
//  Eq. (dequantize) with 127 replaced by 7 in the scale and the clamp).
//
// Storage: two codes per byte, channel 2j in the low nibble and channel 2j+1 in
// the high nibble, two's complement; a row of D channels is D / 2 bytes.
//
// Same streaming shape as the 8-bit kernels: a lane owns 4 adjacent channels
// (one 16-byte fp32 access, one 2-byte code access), wavefronts touch whole
// contiguous row segments, workgroups are small and one-shot.  Rows that cannot
// be accessed that way (D % 4 != 0 or unaligned pointers) take a lane-per-byte path.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

namespace {

// bit pattern whose low 4 bits are the two's-complement 4-bit code of x for divisor s
__device__ __forceinline__ uint32_t nibble_bits(float x, float s) {
  float y = x / s;  // correctly rounded IEEE divide
  y = __builtin_amdgcn_fmed3f(y, -7.0f, 7.0f);
  return __float_as_uint(y + kRoundMagic);
}

// the same from the reciprocal of the divisor (quotient_by: the bits of x / s without the divide sequence)
__device__ __forceinline__ uint32_t nibble_bits_r(float x, double r) {
  float y = quotient_by(x, r);
  y = __builtin_amdgcn_fmed3f(y, -7.0f, 7.0f);
  return __float_as_uint(y + kRoundMagic);
}

// signed 4-bit field i of w -> float (exact) times the channel's scale (one rounding)
__device__ __forceinline__ float dq4(uint32_t w, int i, float s) {
  const int q = (int)(w << (28 - 4 * i)) >> 28;
  return (float)q * s;
}

template <int U, bool NT>
__global__ __launch_bounds__(kMaxBlock) void quantize_int4_kernel(const float* __restrict__ x,
                                                                  const float* __restrict__ scales,
                                                                  uint8_t* __restrict__ packed, int64_t N,
                                                                  int64_t D, int tx_log2, uint32_t ctiles,
                                                                  uint32_t rchunks, int64_t rows_per_chunk,
                                                                  int64_t groups, int64_t f_slab, int64_t p_slab) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * 4;
  const f32x4 sv = *reinterpret_cast<const f32x4*>(scales + it.slab * D + col);
  // With the divide sequence this kernel, which moves 4.5 bytes per element for the arithmetic of 5, ran at
  // 0.82 of the HBM peak on [131072 x 8192]; with the divide-free quotient (same bits) at 0.86.
  const double r0 = reciprocal_of(divisor_of(sv.x)), r1 = reciprocal_of(divisor_of(sv.y)),
               r2 = reciprocal_of(divisor_of(sv.z)), r3 = reciprocal_of(divisor_of(sv.w));
  const int64_t step = (int64_t)it.TY * D;       // elements between the rows a lane visits
  const int64_t pstep = step >> 1;               // the same in packed bytes
  int64_t row = it.row0 + it.ty;
  const float* px = x + it.slab * f_slab + row * D + col;          // slab pitches: fp32 elements, packed bytes
  uint8_t* pc = packed + it.slab * p_slab + ((row * D + col) >> 1);

  auto do_rows = [&](auto nrows_tag) {
    constexpr int R = decltype(nrows_tag)::value;
    f32x4 v[R];
#pragma unroll
    for (int u = 0; u < R; u++) v[u] = ld<NT>(reinterpret_cast<const f32x4*>(px + u * step));
#pragma unroll
    for (int u = 0; u < R; u++) {
      const uint32_t a = nibble_bits_r(v[u].x, r0) & 15u;
      const uint32_t b = nibble_bits_r(v[u].y, r1) & 15u;
      const uint32_t c = nibble_bits_r(v[u].z, r2) & 15u;
      const uint32_t d = nibble_bits_r(v[u].w, r3) & 15u;
      const uint16_t w = (uint16_t)(a | (b << 4) | (c << 8) | (d << 12));
      st<NT>(reinterpret_cast<uint16_t*>(pc + u * pstep), w);
    }
  };
  for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * pstep)
    do_rows(std::integral_constant<int, U>{});
  for (; row < it.row1; row += it.TY, px += step, pc += pstep) do_rows(std::integral_constant<int, 1>{});
}

template <int U, bool NT>
__global__ __launch_bounds__(kMaxBlock) void dequantize_int4_kernel(const uint8_t* __restrict__ packed,
                                                                    const float* __restrict__ scales,
                                                                    float* __restrict__ x_hat, int64_t N,
                                                                    int64_t D, int tx_log2, uint32_t ctiles,
                                                                    uint32_t rchunks, int64_t rows_per_chunk,
                                                                    int64_t groups, int64_t f_slab, int64_t p_slab) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * 4;
  const f32x4 sv = *reinterpret_cast<const f32x4*>(scales + it.slab * D + col);
  const int64_t step = (int64_t)it.TY * D;
  const int64_t pstep = step >> 1;
  int64_t row = it.row0 + it.ty;
  const uint8_t* pc = packed + it.slab * p_slab + ((row * D + col) >> 1);
  float* px = x_hat + it.slab * f_slab + row * D + col;

  auto do_rows = [&](auto nrows_tag) {
    constexpr int R = decltype(nrows_tag)::value;
    uint16_t w[R];
#pragma unroll
    // codes without the streaming hint, as in dequantize_kernel: they may stay in the memory-side cache
    for (int u = 0; u < R; u++) w[u] = ld<false>(reinterpret_cast<const uint16_t*>(pc + u * pstep));
#pragma unroll
    for (int u = 0; u < R; u++) {
      f32x4 o;
      o.x = dq4(w[u], 0, sv.x);
      o.y = dq4(w[u], 1, sv.y);
      o.z = dq4(w[u], 2, sv.z);
      o.w = dq4(w[u], 3, sv.w);
      st<NT>(reinterpret_cast<f32x4*>(px + u * step), o);
    }
  };
  for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * pstep)
    do_rows(std::integral_constant<int, U>{});
  for (; row < it.row1; row += it.TY, px += step, pc += pstep) do_rows(std::integral_constant<int, 1>{});
}

// Lane-per-byte path: a lane owns the two channels of one packed byte.
__global__ __launch_bounds__(kMaxBlock) void quantize_int4_pair_kernel(const float* __restrict__ x,
                                                                       const float* __restrict__ scales,
                                                                       uint8_t* __restrict__ packed, int64_t N,
                                                                       int64_t D, int tx_log2, uint32_t ctiles,
                                                                       uint32_t rchunks, int64_t rows_per_chunk,
                                                                       int64_t groups, int64_t f_slab, int64_t p_slab) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * 2;
  const float s0 = divisor_of(scales[it.slab * D + col]), s1 = divisor_of(scales[it.slab * D + col + 1]);
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  const float* px = x + it.slab * f_slab + row * D + col;          // slab pitches: fp32 elements, packed bytes
  uint8_t* pc = packed + it.slab * p_slab + ((row * D + col) >> 1);
  for (; row < it.row1; row += it.TY, px += step, pc += step >> 1) {
    const uint32_t a = nibble_bits(px[0], s0) & 15u;
    const uint32_t b = nibble_bits(px[1], s1) & 15u;
    *pc = (uint8_t)(a | (b << 4));
  }
}

__global__ __launch_bounds__(kMaxBlock) void dequantize_int4_pair_kernel(const uint8_t* __restrict__ packed,
                                                                         const float* __restrict__ scales,
                                                                         float* __restrict__ x_hat, int64_t N,
                                                                         int64_t D, int tx_log2, uint32_t ctiles,
                                                                         uint32_t rchunks, int64_t rows_per_chunk,
                                                                         int64_t groups, int64_t f_slab, int64_t p_slab) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * 2;
  const float s0 = scales[it.slab * D + col], s1 = scales[it.slab * D + col + 1];
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  const uint8_t* pc = packed + it.slab * p_slab + ((row * D + col) >> 1);
  float* px = x_hat + it.slab * f_slab + row * D + col;
  for (; row < it.row1; row += it.TY, px += step, pc += step >> 1) {
    const uint32_t w = *pc;
    px[0] = dq4(w, 0, s0);
    px[1] = dq4(w, 1, s1);
  }
}

// Launch shape: V = 4 when rows can be moved as 16-byte fp32 / 2-byte code vectors, else 2.
kvq_status int4_tiling(int64_t batch, int64_t N, int64_t D, const void* fp32_ptr, const void* packed,
                       const float* scales, int default_unroll, int default_block, int* U_out, Tiling* t_out) {
  const bool wide = D % 4 == 0 && aligned(fp32_ptr, 16) && aligned(packed, 2) && aligned(scales, 16);
  return stream_tiling(batch, N, D, wide ? 4 : 2, wide, default_unroll, default_block, U_out, t_out);
}

#define KVQ_LAUNCH4(KERNEL, ...)                                                                            \
  do {                                                                                                      \
    const dim3 grid((uint32_t)t.items), block(t.block);                                                     \
    if (t.V == 2)                                                                                           \
      hipLaunchKernelGGL(KERNEL##_pair_kernel, grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2,        \
                         t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, f_slab, p_slab);                                  \
    else if (U == 1 && nt)                                                                                  \
      hipLaunchKernelGGL((KERNEL##_kernel<1, true>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2,  \
                         t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, f_slab, p_slab);                                  \
    else if (U == 2 && nt)                                                                                  \
      hipLaunchKernelGGL((KERNEL##_kernel<2, true>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2,  \
                         t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, f_slab, p_slab);                                  \
    else if (U == 4 && nt)                                                                                  \
      hipLaunchKernelGGL((KERNEL##_kernel<4, true>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2,  \
                         t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, f_slab, p_slab);                                  \
    else if (U == 8 && nt)                                                                                  \
      hipLaunchKernelGGL((KERNEL##_kernel<8, true>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2,  \
                         t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, f_slab, p_slab);                                  \
    else if (U == 1)                                                                                        \
      hipLaunchKernelGGL((KERNEL##_kernel<1, false>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2, \
                         t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, f_slab, p_slab);                                  \
    else if (U == 2)                                                                                        \
      hipLaunchKernelGGL((KERNEL##_kernel<2, false>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2, \
                         t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, f_slab, p_slab);                                  \
    else if (U == 4)                                                                                        \
      hipLaunchKernelGGL((KERNEL##_kernel<4, false>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2, \
                         t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, f_slab, p_slab);                                  \
    else                                                                                                    \
      hipLaunchKernelGGL((KERNEL##_kernel<8, false>), grid, block, 0, stream, __VA_ARGS__, N, D, t.tx_log2, \
                         t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, f_slab, p_slab);                                  \
  } while (0)

}  // namespace

kvq_status launch_quantize_int4(const float* x, const float* scales, uint8_t* packed, int64_t batch, int64_t N,
                                int64_t D, hipStream_t stream) {
  return launch_quantize_int4_strided(x, scales, packed, batch, N, D, N * D, N * D / 2, stream);
}

kvq_status launch_quantize_int4_strided(const float* x, const float* scales, uint8_t* packed, int64_t batch,
                                        int64_t N, int64_t D, int64_t f_slab, int64_t p_slab, hipStream_t stream) {
  int U;
  Tiling t;
  if (kvq_status s = int4_tiling(batch, N, D, x, packed, scales, 4, 512, &U, &t)) return s;
  const bool nt = options().nontemporal != 0;
  KVQ_LAUNCH4(quantize_int4, x, scales, packed);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

kvq_status launch_dequantize_int4(const uint8_t* packed, const float* scales, float* x_hat, int64_t batch,
                                  int64_t N, int64_t D, hipStream_t stream) {
  int U;
  Tiling t;
  // A lane reads only 2 bytes per row, so rows wide enough for it (2048 channels and more) take four rows in
  // flight in 512-lane workgroups: [131072 x 8192] 0.813 -> 0.767 ms, [16384 x 8192] 0.107 -> 0.099 ms.  Narrow
  // rows, which stack several rows per pass, are best with two rows and 256 lanes
  // ([2048 x 4096 x 128] 0.83 against 0.95 ms).
  const bool wide_rows = D >= 2048;
  if (kvq_status s = int4_tiling(batch, N, D, x_hat, packed, scales, wide_rows ? 4 : 2, wide_rows ? 512 : 256, &U, &t))
    return s;
  const int64_t f_slab = N * D, p_slab = N * D / 2;
  const bool nt = options().nontemporal != 0;
  KVQ_LAUNCH4(dequantize_int4, packed, scales, x_hat);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
