// Streaming append: m new tokens join a cache of n_old tokens that is kept
// only as int8 codes and per-channel scales
// (paper: Limitations, "Dynamic quantization" -- scales that adapt during
//  inference; Future Work -- streaming workloads.  The operations are those of
//  Eq. (scale), Eq. (quant_op) and Eq. (dequant_op)).
//
//   cand[d]  = max_t |x_new[t,d]| / 127
//   s_new[d] = cand[d] > s_old[d] ? cand[d] : s_old[d]
//   grown channels (s_new > s_old), cached tokens:  code <- Q(float(code) * s_old ; s_new)
//   new tokens:                                      code  = Q(x_new ; s_new)
// with Q(v; s) = clamp(rint(v / s), -127, 127), 0 for s == 0.
//
// Three steps on the stream, none of which synchronises with the host:
//  1. merge: cand into scales, old scales out to scales_prev.  For a few new
//     tokens (decoding) one kernel does absmax, merge and the quantization of
//     the new rows; for many (a prefill chunk) the batch absmax and quantize
//     kernels do the heavy part around a small elementwise merge.
//  2. requantize: every lane compares old and new scale of its four channels
//     and leaves at once if none grew, so the common step in which no absmax
//     moves costs one pass over the scale arrays.  Lanes that stay walk a long
//     row chunk, rewriting only their own 4-byte code words (a 64-byte line is
//     the unit HBM moves, so a grown channel costs about one read and one
//     write of its slab's rows -- inherent to a token-major cache).
//  3. quantize the new rows behind the cached ones (slab pitch = capacity * D).
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

namespace {

constexpr int kSmallM = 16;            // up to this many new tokens the one-kernel path is used

// int8 code of v for divisor s, in the low byte of the result
__device__ __forceinline__ uint32_t code_bits(float v, float s) {
  float y = v / s;
  y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
  return __float_as_uint(y + kRoundMagic) & 0xffu;
}

__device__ __forceinline__ float merged(float old, float cand) { return cand > old ? cand : old; }

// new tokens come as fp32 (T = float) or as 16-bit patterns (T = f16_tag / bf16_tag), widened exactly
template <typename T>
struct Elem { typedef uint16_t type; };
template <>
struct Elem<float> { typedef float type; };
template <typename T>
__device__ __forceinline__ float load1(const typename Elem<T>::type* p) {
  if constexpr (std::is_same<T, float>::value) return *p;
  else return widen<T>(*p);
}
template <typename T>
__device__ __forceinline__ f32x4 load4(const typename Elem<T>::type* p) {
  if constexpr (std::is_same<T, float>::value) {
    return *reinterpret_cast<const f32x4*>(p);
  } else {
    const u32x2 w = *reinterpret_cast<const u32x2*>(p);
    return f32x4{widen<T>((uint16_t)(w.x & 0xffffu)), widen<T>((uint16_t)(w.x >> 16)),
                 widen<T>((uint16_t)(w.y & 0xffffu)), widen<T>((uint16_t)(w.y >> 16))};
  }
}

// ---- few new tokens: absmax of the new rows, merge, quantize the new rows ----
// One lane per group of V channels of one slab; consecutive lanes own consecutive groups.
template <int V, typename T>
__global__ __launch_bounds__(kBlock) void append_small_kernel(const typename Elem<T>::type* __restrict__ x_new,
                                                              float* __restrict__ scales,
                                                              float* __restrict__ scales_prev,
                                                              int8_t* __restrict__ codes, int64_t lanes,
                                                              int64_t groups, int64_t n_old, int m,
                                                              int64_t capacity, int64_t D) {
  const int64_t id = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (id >= lanes) return;
  const int64_t slab = id / groups;
  const int64_t col = (id - slab * groups) * V;
  const typename Elem<T>::type* px = x_new + slab * m * D + col;
  float mx[V];
#pragma unroll
  for (int i = 0; i < V; i++) mx[i] = 0.0f;
  for (int t = 0; t < m; t++) {
    if constexpr (V == 4) {
      const f32x4 v = load4<T>(px + (int64_t)t * D);
#pragma unroll
      for (int i = 0; i < 4; i++) mx[i] = fmaxf(mx[i], fabsf(v[i]));
    } else {
      mx[0] = fmaxf(mx[0], fabsf(load1<T>(px + (int64_t)t * D)));
    }
  }
  float nw[V];
  float* ps = scales + slab * D + col;
  float* pp = scales_prev + slab * D + col;
  if constexpr (V == 4) {
    const f32x4 old = *reinterpret_cast<const f32x4*>(ps);
    f32x4 n4;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      nw[i] = merged(old[i], mx[i] / 127.0f);
      n4[i] = nw[i];
    }
    *reinterpret_cast<f32x4*>(pp) = old;
    *reinterpret_cast<f32x4*>(ps) = n4;
  } else {
    const float old = *ps;
    nw[0] = merged(old, mx[0] / 127.0f);
    *pp = old;
    *ps = nw[0];
  }
#pragma unroll
  for (int i = 0; i < V; i++) nw[i] = divisor_of(nw[i]);
  int8_t* pc = codes + (slab * capacity + n_old) * D + col;
  for (int t = 0; t < m; t++) {
    if constexpr (V == 4) {
      const f32x4 v = load4<T>(px + (int64_t)t * D);
      const uint32_t w = code_bits(v.x, nw[0]) | (code_bits(v.y, nw[1]) << 8) | (code_bits(v.z, nw[2]) << 16) |
                         (code_bits(v.w, nw[3]) << 24);
      *reinterpret_cast<uint32_t*>(pc + (int64_t)t * D) = w;
    } else {
      pc[(int64_t)t * D] = (int8_t)code_bits(load1<T>(px + (int64_t)t * D), nw[0]);
    }
  }
}

// ---- many new tokens: scales_prev holds cand on entry, the old scales on exit ----
__global__ __launch_bounds__(kBlock) void append_merge_kernel(float* __restrict__ scales,
                                                              float* __restrict__ scales_prev, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= n) return;
  const float old = scales[i], cand = scales_prev[i];
  scales[i] = merged(old, cand);
  scales_prev[i] = old;
}

// ---- cached rows of grown channels ----
// The divide is the divide-free quotient of quotient_by (same bits): with the IEEE sequence this pass is
// bound by the vector ALUs when many channels grow.
__device__ __forceinline__ uint32_t requant_byte(uint32_t word, int b, float s_old, double rcp_new) {
  const int q = (int)(word << (24 - 8 * b)) >> 24;
  const float xh = (float)q * s_old;  // the reconstruction, rounded to fp32 before the divide
  float y = quotient_by(xh, rcp_new);
  y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
  return (__float_as_uint(y + kRoundMagic) & 0xffu) << (8 * b);
}

template <int V, int U>
__global__ __launch_bounds__(kBlock) void append_requant_kernel(int8_t* __restrict__ codes,
                                                                const float* __restrict__ scales,
                                                                const float* __restrict__ scales_prev,
                                                                int64_t n_old, int64_t capacity, int64_t D,
                                                                int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                                int64_t rows_per_chunk, int64_t groups) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, n_old, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * V;
  float so[V], dn[V];
  bool grew[V];
  bool any = false;
#pragma unroll
  for (int i = 0; i < V; i++) {
    so[i] = scales_prev[it.slab * D + col + i];
    const float sn = scales[it.slab * D + col + i];
    grew[i] = sn > so[i];
    any |= grew[i];
    dn[i] = divisor_of(sn);
  }
  if (!any) return;  // no barrier below: lanes leave independently
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  int8_t* pc = codes + (it.slab * capacity + row) * D + col;
  if constexpr (V == 4) {
    double rn[4];
#pragma unroll
    for (int i = 0; i < 4; i++) rn[i] = reciprocal_of(dn[i]);
    uint32_t keep = 0;  // byte mask of the channels that stay as they are
#pragma unroll
    for (int i = 0; i < 4; i++)
      if (!grew[i]) keep |= 0xffu << (8 * i);
    auto do_rows = [&](auto nrows_tag) {
      constexpr int R = decltype(nrows_tag)::value;
      uint32_t w[R];
#pragma unroll
      for (int u = 0; u < R; u++) w[u] = *reinterpret_cast<const uint32_t*>(pc + u * step);
#pragma unroll
      for (int u = 0; u < R; u++) {
        uint32_t r = 0;
#pragma unroll
        for (int i = 0; i < 4; i++) r |= requant_byte(w[u], i, so[i], rn[i]);
        *reinterpret_cast<uint32_t*>(pc + u * step) = (w[u] & keep) | (r & ~keep);
      }
    };
    for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, pc += U * step)
      do_rows(std::integral_constant<int, U>{});
    for (; row < it.row1; row += it.TY, pc += step) do_rows(std::integral_constant<int, 1>{});
  } else {
    for (; row < it.row1; row += it.TY, pc += step) {
      const float xh = (float)(*pc) * so[0];
      *pc = (int8_t)code_bits(xh, dn[0]);
    }
  }
}

}  // namespace

// dtype: KVQ_DTYPE_F32 / F16 / BF16 -- the format of x_new
template <typename T>
static kvq_status append_t(int dtype, const typename Elem<T>::type* x_new, float* scales, float* scales_prev,
                           int8_t* codes, int64_t batch, int64_t n_old, int64_t m, int64_t capacity, int64_t D,
                           hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  // four channels per lane: one 16-byte (fp32) or 8-byte (16-bit) access to the new rows
  const bool wide = D % 4 == 0 && aligned(x_new, 4 * sizeof(typename Elem<T>::type)) && aligned(scales, 16) &&
                    aligned(scales_prev, 16) && aligned(codes, 4);
  const int V = wide ? 4 : 1;
  const int64_t groups = D / V;

  // 1. merge (and, for few tokens, 3. in the same kernel)
  if (m <= kSmallM) {
    const int64_t lanes = batch * groups;
    const int64_t blocks = (lanes + kBlock - 1) / kBlock;
    if (blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
    if (wide)
      hipLaunchKernelGGL((append_small_kernel<4, T>), dim3((uint32_t)blocks), dim3(kBlock), 0, stream, x_new, scales,
                         scales_prev, codes, lanes, groups, n_old, (int)m, capacity, D);
    else
      hipLaunchKernelGGL((append_small_kernel<1, T>), dim3((uint32_t)blocks), dim3(kBlock), 0, stream, x_new, scales,
                         scales_prev, codes, lanes, groups, n_old, (int)m, capacity, D);
    KVQ_HIP(hipGetLastError());
  } else {
    kvq_status s;
    if constexpr (std::is_same<T, float>::value) s = launch_absmax_scales(x_new, scales_prev, batch, m, D, stream);
    else s = launch_absmax_scales_16(dtype, x_new, scales_prev, batch, m, D, stream);
    if (s != KVQ_OK) return s;
    if (kvq_status ms = launch_append_merge(scales, scales_prev, batch * D, stream)) return ms;
  }

  // 2. cached rows of grown channels (rows [0, n_old) only: never the rows written by this call)
  const bool wide_codes = D % 4 == 0 && aligned(scales, 16) && aligned(scales_prev, 16) && aligned(codes, 4);
  if (n_old > 0) {
    constexpr int U = 8;
    Tiling t = make_tiling(batch, n_old, D, wide_codes ? 4 : 1, wide_codes ? U : 1,
                           (int64_t)dev.cus * options().append_blocks_per_cu, kBlock, 0);
    if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
    const dim3 grid((uint32_t)t.items), block(kBlock);
    if (wide_codes)
      hipLaunchKernelGGL((append_requant_kernel<4, U>), grid, block, 0, stream, codes, scales, scales_prev, n_old,
                         capacity, D, t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
    else
      hipLaunchKernelGGL((append_requant_kernel<1, 1>), grid, block, 0, stream, codes, scales, scales_prev, n_old,
                         capacity, D, t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
    KVQ_HIP(hipGetLastError());
  }

  // 3. the new rows
  if (m > kSmallM) {
    if constexpr (std::is_same<T, float>::value)
      return launch_quantize_strided(x_new, scales, codes + n_old * D, batch, m, D, m * D, capacity * D, stream);
    else
      return launch_quantize_16_strided(dtype, x_new, scales, codes + n_old * D, batch, m, D, m * D, capacity * D,
                                        stream);
  }
  return KVQ_OK;
}

kvq_status launch_append_merge(float* scales, float* scales_prev, int64_t n, hipStream_t stream) {
  const int64_t blocks = (n + kBlock - 1) / kBlock;
  if (blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  hipLaunchKernelGGL(append_merge_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0, stream, scales, scales_prev, n);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

kvq_status launch_append(const float* x_new, float* scales, float* scales_prev, int8_t* codes, int64_t batch,
                         int64_t n_old, int64_t m, int64_t capacity, int64_t D, hipStream_t stream) {
  return append_t<float>(KVQ_DTYPE_F32, x_new, scales, scales_prev, codes, batch, n_old, m, capacity, D, stream);
}

kvq_status launch_append_16(int dtype, const void* x_new, float* scales, float* scales_prev, int8_t* codes,
                            int64_t batch, int64_t n_old, int64_t m, int64_t capacity, int64_t D,
                            hipStream_t stream) {
  const uint16_t* p = static_cast<const uint16_t*>(x_new);
  return dtype == KVQ_DTYPE_F16
             ? append_t<f16_tag>(dtype, p, scales, scales_prev, codes, batch, n_old, m, capacity, D, stream)
             : append_t<bf16_tag>(dtype, p, scales, scales_prev, codes, batch, n_old, m, capacity, D, stream);
}

}  // namespace kvq
