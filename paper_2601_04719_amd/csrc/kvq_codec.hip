// Quantize and dequantize kernels
// (paper: Eq. (quantize)/(quant_op) with the clamp of the Method section;
//  Eq. (dequantize)/(dequant_op)).
//
// Both are pure streams (4 B in + 1 B out, or 1 B in + 4 B out per element),
// so the layout is chosen for the memory system: a lane owns V adjacent
// channels (V = 16: four 16-byte fp32 accesses and one 16-byte code access),
// keeps their scales in registers for its whole walk down the rows, and has
// U rows in flight.  The paper's fastest variant moves 4 codes per thread and
// reloads the scales for every element; its shared-memory staging of scales
// has no counterpart here because nothing is re-read.
//
// Rounding is done without a convert instruction: after the clamp to
// [-127,127], adding 1.5*2^23 rounds to the nearest integer with ties to even
// (the sum lies in [2^23,2^24) where the spacing is 1 and 1.5*2^23 is even) and
// leaves the two's-complement code in the low byte of the sum's bit pattern.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

constexpr float kMagic = 12582912.0f;  // 1.5 * 2^23

// Distance from a .5 tie below which the reciprocal-multiply quotient may round
// differently from the correctly rounded quotient: |x*r - fl(x/s)| <=
// 1.5*2^-23 |x/s| < 2^-14 whenever |x/s| < 256, and larger quotients clamp to
// +-127 either way.
constexpr float kTieBand = 0.5f - 6.103515625e-05f;  // 0.5 - 2^-14

struct LaneScale {
  float s;  // divisor: the scale, or +inf for a zero scale (x/inf = 0 -> code 0)
  float r;  // multiplier for the fast path: 1/s, 0 for a zero scale, NaN if 1/s is not safely normal
};

__device__ __forceinline__ LaneScale prepare_scale(float s) {
  LaneScale ls;
  if (s == 0.0f) {
    ls.s = __builtin_inff();
    ls.r = 0.0f;
  } else {
    ls.s = s;
    const float a = fabsf(s);
    ls.r = (a >= 0x1p-100f && a <= 0x1p100f) ? 1.0f / s : __builtin_nanf("");
  }
  return ls;
}

// Returns the float whose low byte is the int8 code of x under scale ls.
template <bool EXACT>
__device__ __forceinline__ float code_as_float(float x, const LaneScale& ls) {
  float y;
  if constexpr (EXACT) {
    y = x / ls.s;  // correctly rounded IEEE divide
  } else {
    y = x * ls.r;
    const float f = fabsf(y - rintf(y));
    if (!(f < kTieBand)) y = x / ls.s;  // near a tie (or unsafe scale): decide with the true quotient
  }
  y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
  return y + kMagic;
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
template <int V, int U, bool NT, bool EXACT>
__global__ __launch_bounds__(kBlock) void quantize_kernel(const float* __restrict__ x,
                                                          const float* __restrict__ scales,
                                                          int8_t* __restrict__ codes, int64_t N, int64_t D,
                                                          int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                          int64_t rows_per_chunk, int64_t groups) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * V;
  LaneScale ls[V];
  {
    const float* sp = scales + it.slab * D + col;
#pragma unroll
    for (int i = 0; i < V; i++) ls[i] = prepare_scale(sp[i]);
  }
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  const float* px = x + (it.slab * N + row) * D + col;
  int8_t* pc = codes + (it.slab * N + row) * D + col;

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
          const float a = code_as_float<EXACT>(v[u][w].x, ls[4 * w + 0]);
          const float b = code_as_float<EXACT>(v[u][w].y, ls[4 * w + 1]);
          const float cc = code_as_float<EXACT>(v[u][w].z, ls[4 * w + 2]);
          const float d = code_as_float<EXACT>(v[u][w].w, ls[4 * w + 3]);
          set_word<V>(c, w, pack4(a, b, cc, d));
        }
        st<NT>(reinterpret_cast<cvec*>(pc + u * step), c);
      }
    };
    for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * step)
      do_rows(std::integral_constant<int, U>{});
    for (; row < it.row1; row += it.TY, px += step, pc += step) do_rows(std::integral_constant<int, 1>{});
  } else {
    for (; row < it.row1; row += it.TY, px += step, pc += step) {
      const float a = code_as_float<EXACT>(*px, ls[0]);
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

template <int V, int U, bool NT>
__global__ __launch_bounds__(kBlock) void dequantize_kernel(const int8_t* __restrict__ codes,
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
#pragma unroll
    for (int i = 0; i < V; i++) s[i] = sp[i];
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
      for (int u = 0; u < R; u++) c[u] = ld<NT>(reinterpret_cast<const cvec*>(pc + u * step));
#pragma unroll
      for (int u = 0; u < R; u++)
#pragma unroll
        for (int w = 0; w < W; w++) {
          const uint32_t word = word_of<V>(c[u], w);
          f32x4 o;
          o.x = dq(word, 0, s[4 * w + 0]);
          o.y = dq(word, 1, s[4 * w + 1]);
          o.z = dq(word, 2, s[4 * w + 2]);
          o.w = dq(word, 3, s[4 * w + 3]);
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
                           const Tiling& t, bool nt, bool exact, hipStream_t stream) {
  const dim3 grid((uint32_t)t.items), block(kBlock);
#define KVQ_LAUNCH_Q(NT_, EX_)                                                                           \
  hipLaunchKernelGGL((quantize_kernel<V, U, NT_, EX_>), grid, block, 0, stream, x, scales, codes, N, D, \
                     t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups)
  if (nt && exact) KVQ_LAUNCH_Q(true, true);
  else if (nt) KVQ_LAUNCH_Q(true, false);
  else if (exact) KVQ_LAUNCH_Q(false, true);
  else KVQ_LAUNCH_Q(false, false);
#undef KVQ_LAUNCH_Q
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

template <int V, int U>
static kvq_status launch_d(const int8_t* codes, const float* scales, float* x_hat, int64_t N, int64_t D,
                           const Tiling& t, bool nt, hipStream_t stream) {
  const dim3 grid((uint32_t)t.items), block(kBlock);
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
  KVQ_CASE(16, 1); KVQ_CASE(16, 2); KVQ_CASE(16, 4);
  KVQ_CASE(8, 1); KVQ_CASE(8, 2); KVQ_CASE(8, 4);
  KVQ_CASE(4, 1); KVQ_CASE(4, 2); KVQ_CASE(4, 4);
#undef KVQ_CASE
  return f(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{});
}

kvq_status launch_quantize(const float* x, const float* scales, int8_t* codes, int64_t batch, int64_t N,
                           int64_t D, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  const Options o = options();
  const int V = pick_width(D, x, codes, o.codec_width);
  const int U = V == 1 ? 1 : o.codec_unroll;
  const Tiling t = make_tiling(batch, N, D, V, U, (int64_t)dev.cus * o.blocks_per_cu);
  if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
  return dispatch_vu(V, U, [&](auto v, auto u) {
    return launch_q<decltype(v)::value, decltype(u)::value>(x, scales, codes, N, D, t, o.nontemporal != 0,
                                                            o.exact_div_only != 0, stream);
  });
}

kvq_status launch_dequantize(const int8_t* codes, const float* scales, float* x_hat, int64_t batch,
                             int64_t N, int64_t D, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  const Options o = options();
  const int V = pick_width(D, x_hat, codes, o.codec_width);
  const int U = V == 1 ? 1 : o.codec_unroll;
  const Tiling t = make_tiling(batch, N, D, V, U, (int64_t)dev.cus * o.blocks_per_cu);
  if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
  return dispatch_vu(V, U, [&](auto v, auto u) {
    return launch_d<decltype(v)::value, decltype(u)::value>(codes, scales, x_hat, N, D, t,
                                                            o.nontemporal != 0, stream);
  });
}

}  // namespace kvq
