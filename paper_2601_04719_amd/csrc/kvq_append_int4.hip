// Streaming append onto a 4-bit cache: the method of kvq_append with the integer range [-7, 7]
// and two codes per byte
// (paper: Limitations, "Dynamic quantization" and "Lower bit-widths"; Eq. (scale), Eq. (quant_op),
//  Eq. (dequant_op) with 127 replaced by 7).
//
//   cand[d]  = max_t |x_new[t,d]| / 7
//   s_new[d] = cand[d] > s_old[d] ? cand[d] : s_old[d]
//   grown channels, cached tokens:  code <- Q7(float(code) * s_old ; s_new)
//   new tokens:                      code  = Q7(x_new ; s_new)
// with Q7(v; s) = clamp(rint(v / s), -7, 7), 0 for s == 0; channel 2j in the low and 2j+1 in the
// high nibble of byte j of a row.
//
// Same three steps as the 8-bit append.  A lane owns 4 adjacent channels -- one 16-bit word of
// every packed row -- or, where rows or pointers do not allow that, the 2 channels of one byte.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

namespace {

constexpr int kSmallM4 = 16;  // up to this many new tokens the one-kernel path is used

// two's-complement 4-bit code of v for divisor s, in the low nibble of the result
__device__ __forceinline__ uint32_t nibble_of(float v, float s) {
  float y = v / s;  // correctly rounded IEEE divide
  y = __builtin_amdgcn_fmed3f(y, -7.0f, 7.0f);
  return __float_as_uint(y + kRoundMagic) & 15u;
}

__device__ __forceinline__ float larger(float old, float cand) { return cand > old ? cand : old; }

// the V codes of a lane's channels for one row, packed low nibble first
template <int V>
__device__ __forceinline__ uint32_t pack_row(const float (&v)[V], const float (&div)[V]) {
  uint32_t w = 0;
#pragma unroll
  for (int i = 0; i < V; i++) w |= nibble_of(v[i], div[i]) << (4 * i);
  return w;
}

template <int V>
__device__ __forceinline__ void load_row(const float* p, float (&v)[V]) {
  if constexpr (V == 4) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  } else {
    v[0] = p[0];
    v[1] = p[1];
  }
}

template <int V>
__device__ __forceinline__ void store_codes(uint8_t* p, uint32_t w) {
  if constexpr (V == 4) *reinterpret_cast<uint16_t*>(p) = (uint16_t)w;
  else *p = (uint8_t)w;
}

template <int V>
__device__ __forceinline__ uint32_t load_codes(const uint8_t* p) {
  if constexpr (V == 4) return *reinterpret_cast<const uint16_t*>(p);
  else return *p;
}

// ---- few new tokens: absmax of the new rows, merge, quantize the new rows ----
// One lane per group of V channels of one slab; consecutive lanes own consecutive groups.
template <int V>
__global__ __launch_bounds__(kBlock) void append4_small_kernel(const float* __restrict__ x_new,
                                                               float* __restrict__ scales,
                                                               float* __restrict__ scales_prev,
                                                               uint8_t* __restrict__ packed, int64_t lanes,
                                                               int64_t groups, int64_t n_old, int m,
                                                               int64_t capacity, int64_t D) {
  const int64_t id = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (id >= lanes) return;
  const int64_t slab = id / groups;
  const int64_t col = (id - slab * groups) * V;
  const float* px = x_new + slab * m * D + col;
  float mx[V];
#pragma unroll
  for (int i = 0; i < V; i++) mx[i] = 0.0f;
  for (int t = 0; t < m; t++) {
    float v[V];
    load_row<V>(px + (int64_t)t * D, v);
#pragma unroll
    for (int i = 0; i < V; i++) mx[i] = fmaxf(mx[i], fabsf(v[i]));
  }
  float div[V];
  float* ps = scales + slab * D + col;
  float* pp = scales_prev + slab * D + col;
#pragma unroll
  for (int i = 0; i < V; i++) {
    const float old = ps[i];
    const float nw = larger(old, mx[i] / 7.0f);
    pp[i] = old;
    ps[i] = nw;
    div[i] = divisor_of(nw);
  }
  uint8_t* pc = packed + (((slab * capacity + n_old) * D + col) >> 1);
  for (int t = 0; t < m; t++) {
    float v[V];
    load_row<V>(px + (int64_t)t * D, v);
    store_codes<V>(pc + (((int64_t)t * D) >> 1), pack_row<V>(v, div));
  }
}

// ---- cached rows of grown channels ----
template <int V, int U>
__global__ __launch_bounds__(kBlock) void append4_requant_kernel(uint8_t* __restrict__ packed,
                                                                 const float* __restrict__ scales,
                                                                 const float* __restrict__ scales_prev,
                                                                 int64_t n_old, int64_t capacity, int64_t D,
                                                                 int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                                 int64_t rows_per_chunk, int64_t groups) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, n_old, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * V;
  float so[V], dn[V];
  uint32_t keep = 0;  // nibble mask of the channels that stay as they are
  bool any = false;
#pragma unroll
  for (int i = 0; i < V; i++) {
    so[i] = scales_prev[it.slab * D + col + i];
    const float sn = scales[it.slab * D + col + i];
    if (sn > so[i]) any = true;
    else keep |= 15u << (4 * i);
    dn[i] = divisor_of(sn);
  }
  if (!any) return;  // no barrier below: lanes leave independently
  double rn[V];  // the divide below as the divide-free quotient of quotient_by (same bits)
#pragma unroll
  for (int i = 0; i < V; i++) rn[i] = reciprocal_of(dn[i]);
  const int64_t pstep = ((int64_t)it.TY * D) >> 1;  // packed bytes between the rows a lane visits
  int64_t row = it.row0 + it.ty;
  uint8_t* pc = packed + (((it.slab * capacity + row) * D + col) >> 1);
  auto do_rows = [&](auto nrows_tag) {
    constexpr int R = decltype(nrows_tag)::value;
    uint32_t w[R];
#pragma unroll
    for (int u = 0; u < R; u++) w[u] = load_codes<V>(pc + u * pstep);
#pragma unroll
    for (int u = 0; u < R; u++) {
      uint32_t r = 0;
#pragma unroll
      for (int i = 0; i < V; i++) {
        const int q = (int)(w[u] << (28 - 4 * i)) >> 28;
        const float xh = (float)q * so[i];  // the reconstruction, rounded to fp32 before the divide
        float y = quotient_by(xh, rn[i]);
        y = __builtin_amdgcn_fmed3f(y, -7.0f, 7.0f);
        r |= (__float_as_uint(y + kRoundMagic) & 15u) << (4 * i);
      }
      store_codes<V>(pc + u * pstep, (w[u] & keep) | (r & ~keep));
    }
  };
  for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, pc += U * pstep)
    do_rows(std::integral_constant<int, U>{});
  for (; row < it.row1; row += it.TY, pc += pstep) do_rows(std::integral_constant<int, 1>{});
}

}  // namespace

kvq_status launch_append_int4(const float* x_new, float* scales, float* scales_prev, uint8_t* packed, int64_t batch,
                              int64_t n_old, int64_t m, int64_t capacity, int64_t D, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  // four channels per lane: 16-byte access to the new rows, 2-byte access to the packed rows
  const bool wide_codes = D % 4 == 0 && aligned(packed, 2);
  const bool wide = wide_codes && aligned(x_new, 16);

  // 1. merge (and, for few tokens, 3. in the same kernel)
  if (m <= kSmallM4) {
    const int V = wide ? 4 : 2;
    const int64_t groups = D / V;
    const int64_t lanes = batch * groups;
    const int64_t blocks = (lanes + kBlock - 1) / kBlock;
    if (blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
    if (wide)
      hipLaunchKernelGGL(append4_small_kernel<4>, dim3((uint32_t)blocks), dim3(kBlock), 0, stream, x_new, scales,
                         scales_prev, packed, lanes, groups, n_old, (int)m, capacity, D);
    else
      hipLaunchKernelGGL(append4_small_kernel<2>, dim3((uint32_t)blocks), dim3(kBlock), 0, stream, x_new, scales,
                         scales_prev, packed, lanes, groups, n_old, (int)m, capacity, D);
    KVQ_HIP(hipGetLastError());
  } else {
    if (kvq_status s = launch_absmax_scales(x_new, scales_prev, batch, m, D, stream, 7.0f)) return s;
    if (kvq_status s = launch_append_merge(scales, scales_prev, batch * D, stream)) return s;
  }

  // 2. cached rows of grown channels (rows [0, n_old) only: never the rows written by this call)
  if (n_old > 0) {
    constexpr int U = 8;
    const int V = wide_codes ? 4 : 2;
    Tiling t = make_tiling(batch, n_old, D, V, U, (int64_t)dev.cus * options().append_blocks_per_cu, kBlock, 0);
    if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
    const dim3 grid((uint32_t)t.items), block(kBlock);
    if (wide_codes)
      hipLaunchKernelGGL((append4_requant_kernel<4, U>), grid, block, 0, stream, packed, scales, scales_prev, n_old,
                         capacity, D, t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
    else
      hipLaunchKernelGGL((append4_requant_kernel<2, U>), grid, block, 0, stream, packed, scales, scales_prev, n_old,
                         capacity, D, t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
    KVQ_HIP(hipGetLastError());
  }

  // 3. the new rows
  if (m > kSmallM4)
    return launch_quantize_int4_strided(x_new, scales, packed + ((n_old * D) >> 1), batch, m, D, m * D,
                                        (capacity * D) >> 1, stream);
  return KVQ_OK;
}

}  // namespace kvq
