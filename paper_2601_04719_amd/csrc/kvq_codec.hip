// Quantize and dequantize kernels
// (paper: Eq. (quantize)/(quant_op) with the clamp of the Method section;
//  Eq. (dequantize)/(dequant_op)).
//
// Both are pure streams (4 B in + 1 B out, or 1 B in + 4 B out per element),
// so everything here is chosen for the memory system, by measurement:
//  - a lane owns V = 4 adjacent channels: one 16-byte fp32 access and one
//    4-byte code access, so every memory instruction of a wavefront covers one
//    contiguous 1 KiB (fp32) or 256 B (codes) segment.  Wider lanes (V = 8, 16:
//    several 16-byte accesses per lane, 64-byte lane pitch) are kept as
//    selectable variants; they are slower because each instruction then touches
//    a quarter of many cache lines.
//  - workgroups are small and one-shot: each handles U rows of its column tile
//    and exits, and the hardware dispatcher hands tiles out in address order,
//    which keeps the set of DRAM pages in use compact.  Persistent grid-stride
//    loops measured 10-20 % slower.  Defaults from interleaved sweeps over
//    D = 1024..8192: quantize 512 lanes x 4 rows, dequantize 256 lanes x 2 rows.
//  - the scales of a lane are read once per workgroup (they stay in L2); the
//    paper's shared-memory staging of scales has no counterpart because nothing
//    is re-read.
//
// Rounding is done without a convert instruction: after the clamp to
// [-127,127], adding kRoundMagic leaves the int8 code in the low byte of the sum.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

// Returns the float whose low byte is the int8 code of x for divisor s.
__device__ __forceinline__ float code_as_float(float x, float s) {
  float y = x / s;  // correctly rounded IEEE divide (the full v_div_scale/fmas/fixup sequence)
  y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
  return y + kRoundMagic;
}

// low bytes of four words -> one word (a in byte 0 ... d in byte 3)
__device__ __forceinline__ uint32_t pack4(float a, float b, float c, float d) {
  const uint32_t lo = __builtin_amdgcn_perm(__float_as_uint(b), __float_as_uint(a), 0x0c0c0400u);
  const uint32_t hi = __builtin_amdgcn_perm(__float_as_uint(d), __float_as_uint(c), 0x0c0c0400u);
  return __builtin_amdgcn_perm(hi, lo, 0x05040100u);
}

template <int V>
struct CodeVec;
template <>
struct CodeVec<4> { typedef uint32_t type; };
template <>
struct CodeVec<8> { typedef u32x2 type; };
template <>
struct CodeVec<16> { typedef u32x4 type; };

template <int V>
__device__ __forceinline__ uint32_t word_of(const typename CodeVec<V>::type& c, int w) {
  if constexpr (V == 4) return c;
  else return c[w];
}
template <int V>
__device__ __forceinline__ void set_word(typename CodeVec<V>::type& c, int w, uint32_t v) {
  if constexpr (V == 4) c = v;
  else c[w] = v;
}

// ------------------------------------------------------------------ quantize
// MATH = false gives the no-math streaming probe: same loads and stores, codes replaced by a bit mix.
template <int V, int U, bool NT, bool MATH = true>
__global__ __launch_bounds__(kMaxBlock) void quantize_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ scales,
                                                          int8_t* __restrict__ codes, int64_t N, int64_t D,
                                                          int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                          int64_t rows_per_chunk, int64_t groups,
                                                          int64_t x_slab, int64_t c_slab) {
  // x_slab / c_slab: elements between consecutive slabs of x and of codes (N * D when both are dense)
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * V;
  float ls[V];
  {
    const float* sp = scales + it.slab * D + col;
    if constexpr (V >= 4) {
#pragma unroll
      for (int w = 0; w < V / 4; w++) {
        const f32x4 sv = *(reinterpret_cast<const f32x4*>(sp) + w);
#pragma unroll
        for (int i = 0; i < 4; i++) ls[4 * w + i] = divisor_of(sv[i]);
      }
    } else {
      ls[0] = divisor_of(sp[0]);
    }
  }
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  const float* px = x + it.slab * x_slab + row * D + col;
  int8_t* pc = codes + it.slab * c_slab + row * D + col;

  if constexpr (V >= 4) {
    typedef typename CodeVec<V>::type cvec;
    constexpr int W = V / 4;
    auto do_rows = [&](auto nrows_tag) {
      constexpr int R = decltype(nrows_tag)::value;
      f32x4 v[R][W];
#pragma unroll
      for (int u = 0; u < R; u++)
#pragma unroll
        for (int w = 0; w < W; w++) v[u][w] = ld<NT>(reinterpret_cast<const f32x4*>(px + u * step) + w);
#pragma unroll
      for (int u = 0; u < R; u++) {
        cvec c;
#pragma unroll
        for (int w = 0; w < W; w++) {
          if constexpr (MATH) {
            const float a = code_as_float(v[u][w].x, ls[4 * w + 0]);
            const float b = code_as_float(v[u][w].y, ls[4 * w + 1]);
            const float cc = code_as_float(v[u][w].z, ls[4 * w + 2]);
            const float d = code_as_float(v[u][w].w, ls[4 * w + 3]);
            set_word<V>(c, w, pack4(a, b, cc, d));
          } else {
            set_word<V>(c, w, __float_as_uint(v[u][w].x) ^ __float_as_uint(v[u][w].y) ^ __float_as_uint(v[u][w].z) ^
                                  __float_as_uint(v[u][w].w) ^ __float_as_uint(ls[4 * w]));
          }
        }
        st<NT>(reinterpret_cast<cvec*>(pc + u * step), c);
      }
    };
    for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * step)
      do_rows(std::integral_constant<int, U>{});
    for (; row < it.row1; row += it.TY, px += step, pc += step) do_rows(std::integral_constant<int, 1>{});
  } else {
    for (; row < it.row1; row += it.TY, px += step, pc += step) {
      const float a = code_as_float(*px, ls[0]);
      *pc = (int8_t)(__float_as_uint(a) & 0xffu);
    }
  }
}

// ---------------------------------------------------------------- dequantize
// signed byte b of a word -> float (exact), times the channel's scale (one rounding)
__device__ __forceinline__ float dq(uint32_t word, int b, float s) {
  const int q = (int)(word << (24 - 8 * b)) >> 24;
  return (float)q * s;
}

template <int V, int U, bool NT, bool MATH = true>
__global__ __launch_bounds__(kMaxBlock) void dequantize_kernel(const int8_t* __restrict__ codes,
                                                            const float* __restrict__ scales,
                                                            float* __restrict__ x_hat, int64_t N, int64_t D,
                                                            int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                            int64_t rows_per_chunk, int64_t groups) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * V;
  float s[V];
  {
    const float* sp = scales + it.slab * D + col;
    if constexpr (V >= 4) {
#pragma unroll
      for (int w = 0; w < V / 4; w++) {
        const f32x4 sv = *(reinterpret_cast<const f32x4*>(sp) + w);
#pragma unroll
        for (int i = 0; i < 4; i++) s[4 * w + i] = sv[i];
      }
    } else {
      s[0] = sp[0];
    }
  }
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  const int8_t* pc = codes + (it.slab * N + row) * D + col;
  float* px = x_hat + (it.slab * N + row) * D + col;

  if constexpr (V >= 4) {
    typedef typename CodeVec<V>::type cvec;
    constexpr int W = V / 4;
    auto do_rows = [&](auto nrows_tag) {
      constexpr int R = decltype(nrows_tag)::value;
      cvec c[R];
#pragma unroll
      // The codes are loaded without the streaming hint, whatever NT says for the stores: they are the part of
      // this call that a serving loop reads again (every pass over the cache), a quarter of the bytes, and left
      // to the caches they stay in the 256 MiB memory-side cache where they fit -- HBM then only has the
      // fp32 stream to write ([16384 x 8192] called again and again: 0.106 -> 0.097 ms, [64 x 4096 x 1024]
      // 0.213 -> 0.189; with six buffer pairs in rotation, so that nothing is found again, 0.105 -> 0.108;
      // [131072 x 8192], whose codes are four times the cache: 0.800 -> 0.790).
      for (int u = 0; u < R; u++) c[u] = ld<false>(reinterpret_cast<const cvec*>(pc + u * step));
#pragma unroll
      for (int u = 0; u < R; u++)
#pragma unroll
        for (int w = 0; w < W; w++) {
          const uint32_t word = word_of<V>(c[u], w);
          f32x4 o;
          if constexpr (MATH) {
            o.x = dq(word, 0, s[4 * w + 0]);
            o.y = dq(word, 1, s[4 * w + 1]);
            o.z = dq(word, 2, s[4 * w + 2]);
            o.w = dq(word, 3, s[4 * w + 3]);
          } else {
            o.x = __uint_as_float(word);
            o.y = s[4 * w + 1];
            o.z = __uint_as_float(word >> 8);
            o.w = s[4 * w + 3];
          }
          st<NT>(reinterpret_cast<f32x4*>(px + u * step) + w, o);
        }
    };
    for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * step)
      do_rows(std::integral_constant<int, U>{});
    for (; row < it.row1; row += it.TY, px += step, pc += step) do_rows(std::integral_constant<int, 1>{});
  } else {
    for (; row < it.row1; row += it.TY, px += step, pc += step) *px = (float)(*pc) * s[0];
  }
}

// ----------------------------------------------------------------- launchers
template <int V, int U>
static kvq_status launch_q(const float* x, const float* scales, int8_t* codes, int64_t N, int64_t D,
                           const Tiling& t, bool nt, hipStream_t stream, int64_t x_slab, int64_t c_slab) {
  const dim3 grid((uint32_t)t.items), block(t.block);
  if (nt)
    hipLaunchKernelGGL((quantize_kernel<V, U, true>), grid, block, 0, stream, x, scales, codes, N, D, t.tx_log2,
                       t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, x_slab, c_slab);
  else
    hipLaunchKernelGGL((quantize_kernel<V, U, false>), grid, block, 0, stream, x, scales, codes, N, D, t.tx_log2,
                       t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, x_slab, c_slab);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

template <int V, int U>
static kvq_status launch_d(const int8_t* codes, const float* scales, float* x_hat, int64_t N, int64_t D,
                           const Tiling& t, bool nt, hipStream_t stream) {
  const dim3 grid((uint32_t)t.items), block(t.block);
  if (nt)
    hipLaunchKernelGGL((dequantize_kernel<V, U, true>), grid, block, 0, stream, codes, scales, x_hat, N, D,
                       t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
  else
    hipLaunchKernelGGL((dequantize_kernel<V, U, false>), grid, block, 0, stream, codes, scales, x_hat, N, D,
                       t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

template <typename F>
static kvq_status dispatch_vu(int V, int U, F&& f) {
#define KVQ_CASE(V_, U_) \
  if (V == V_ && U == U_) return f(std::integral_constant<int, V_>{}, std::integral_constant<int, U_>{})
  KVQ_CASE(4, 1); KVQ_CASE(4, 2); KVQ_CASE(4, 4); KVQ_CASE(4, 8);
  KVQ_CASE(8, 1); KVQ_CASE(8, 2); KVQ_CASE(8, 4);
  KVQ_CASE(16, 1); KVQ_CASE(16, 2); KVQ_CASE(16, 4);
#undef KVQ_CASE
  return f(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{});
}

// Launch shape of a codec kernel.  Vector lanes need the scale rows 16-byte
// aligned too (batch > 1 with D % 4 == 0 keeps every slab's scales aligned).
static kvq_status codec_tiling(int64_t batch, int64_t N, int64_t D, const void* fp32_ptr, const void* int8_ptr,
                               const float* scales, int default_unroll, int default_block, int* U_out,
                               Tiling* t_out) {
  int V = pick_width(D, fp32_ptr, int8_ptr, options().codec_width);
  if (V > 1 && !aligned(scales, 16)) V = 1;
  return stream_tiling(batch, N, D, V, V > 1, default_unroll, default_block, U_out, t_out);
}

kvq_status launch_quantize(const float* x, const float* scales, int8_t* codes, int64_t batch, int64_t N,
                           int64_t D, hipStream_t stream) {
  return launch_quantize_strided(x, scales, codes, batch, N, D, N * D, N * D, stream);
}

kvq_status launch_quantize_strided(const float* x, const float* scales, int8_t* codes, int64_t batch, int64_t N,
                                   int64_t D, int64_t x_slab, int64_t c_slab, hipStream_t stream) {
  int U;
  Tiling t;
  // both slab pitches are multiples of D, so the alignment of row 0 of slab 0 decides for all rows
  if (kvq_status s = codec_tiling(batch, N, D, x, codes, scales, kQuantUnroll, kQuantBlock, &U, &t)) return s;
  const bool nt = options().nontemporal != 0;
  return dispatch_vu(t.V, U, [&](auto v, auto u) {
    return launch_q<decltype(v)::value, decltype(u)::value>(x, scales, codes, N, D, t, nt, stream, x_slab, c_slab);
  });
}

kvq_status launch_dequantize(const int8_t* codes, const float* scales, float* x_hat, int64_t batch,
                             int64_t N, int64_t D, hipStream_t stream) {
  int U;
  Tiling t;
  if (kvq_status s = codec_tiling(batch, N, D, x_hat, codes, scales, kDequantUnroll, dequant_block_for(D), &U, &t)) return s;
  const bool nt = options().nontemporal != 0;
  return dispatch_vu(t.V, U, [&](auto v, auto u) {
    return launch_d<decltype(v)::value, decltype(u)::value>(codes, scales, x_hat, N, D, t, nt, stream);
  });
}

// No-math probes with the production launch shape (default options): mode 2 = the quantize traffic
// (4 B in, 1 B out), mode 3 = the dequantize traffic (1 B in, 4 B out).
kvq_status launch_probe_codec(int mode, const float* src_f32, float* dst_f32, const int8_t* src_i8,
                              int8_t* dst_i8, const float* scales, int64_t batch, int64_t N, int64_t D,
                              hipStream_t stream) {
  int U;
  Tiling t;
  if (mode == 2) {
    if (kvq_status s = codec_tiling(batch, N, D, src_f32, dst_i8, scales, 4, 512, &U, &t)) return s;
    if (t.V != 4 || U != 4) return KVQ_ERR_ARG;
    hipLaunchKernelGGL((quantize_kernel<4, 4, true, false>), dim3((uint32_t)t.items), dim3(t.block), 0, stream,
                       src_f32, scales, dst_i8, N, D, t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups,
                       N * D, N * D);
  } else {
    if (kvq_status s = codec_tiling(batch, N, D, dst_f32, src_i8, scales, 2, dequant_block_for(D), &U, &t)) return s;
    if (t.V != 4 || U != 2) return KVQ_ERR_ARG;
    hipLaunchKernelGGL((dequantize_kernel<4, 2, true, false>), dim3((uint32_t)t.items), dim3(t.block), 0, stream,
                       src_i8, scales, dst_f32, N, D, t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
  }
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
