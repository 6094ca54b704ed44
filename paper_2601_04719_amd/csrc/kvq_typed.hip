// The same scale computation, quantization and dequantization for fp16 and bf16 matrices
// (paper: "Memory Bottleneck in LLM Inference" notes that real caches are kept in 16-bit formats;
//  the arithmetic is that of Eq. (scale_compute), Eq. (quant_op), Eq. (dequant_op)).
//
// A 16-bit value converts to fp32 exactly, so scales and codes are what the fp32 path would give
// for the widened matrix; dequantization forms (float)code * scale in fp32 and rounds it once more,
// to nearest even, into the 16-bit format.  Traffic is 2 B in + 1 B out per element (or the
// reverse).  A lane owns 8 adjacent channels: one 16-byte access on the 16-bit side, one 8-byte
// access on the code side, both contiguous across a wavefront.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

template <typename T>
__device__ __forceinline__ void widen8(const u16x8& raw, float (&out)[8]) {
#pragma unroll
  for (int i = 0; i < 8; i++) out[i] = widen<T>(raw[i]);
}


// int8 code of x for the divisor div, by the plain IEEE divide (the scalar path)
__device__ __forceinline__ uint32_t code_byte(float x, float div) {
  float y = x / div;
  y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
  return __float_as_uint(y + kRoundMagic) & 0xffu;
}

// int8 code of x by the divide-free quotient (see quotient_by): what the vector kernel runs, because with
// the divide sequence it was bound by the vector ALUs, not by HBM.
// Tried on top of it and not kept: an fp32-only fast form (y = x * fl(1 / div), exact unless y lies within
// 2^-15 of a half-integer, with the exact form as the fall-back for the wavefront).  It is correct, but
// 16-bit inputs put near-ties everywhere: a value that is exactly half the column's absmax gives a quotient
// within an ulp of 63.5, and such values recur because a binade holds only 128 (bf16) or 1024 (fp16)
// different numbers -- 1.3e-3 of all bf16 elements of a Gaussian matrix, so every second wavefront piece
// took the fall-back and the kernel ran at 0.64-0.78 ms instead of 0.50 ms on [131072 x 8192].
__device__ __forceinline__ uint32_t code_byte_r(float x, double r) {
  float y = quotient_by(x, r);
  y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
  return __float_as_uint(y + kRoundMagic) & 0xffu;
}

// ---- absmax --------------------------------------------------------------------------------
// V = 8 (vector) or 1 (scalar); J column groups per lane, TX groups apart (see the fp32 kernel)
template <typename T, int V, int J, int U>
__global__ __launch_bounds__(kBlock) void absmax16_kernel(const uint16_t* __restrict__ x, float* __restrict__ dst,
                                                          int64_t chunk_stride, int64_t N, int64_t D, int tx_log2,
                                                          uint32_t ctiles, uint32_t rchunks, int64_t rows_per_chunk,
                                                          int64_t groups) {
  __shared__ float red[J == 1 ? kBlock * V : 1];
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  const int TX = 1 << tx_log2;
  const int tx = threadIdx.x & (TX - 1);
  const int64_t group0 = (it.group - tx) * J + tx;
  float m[J][V];
  bool act[J];
#pragma unroll
  for (int j = 0; j < J; j++) {
    act[j] = group0 + (int64_t)j * TX < groups;
#pragma unroll
    for (int i = 0; i < V; i++) m[j][i] = 0.0f;
  }
  if (act[0]) {
    const int64_t step = (int64_t)it.TY * D;
    int64_t row = it.row0 + it.ty;
    const uint16_t* p = x + (it.slab * N + row) * D + group0 * V;
    if constexpr (V == 8) {
      auto do_rows = [&](auto tag) {
        constexpr int R = decltype(tag)::value;
        u16x8 v[R][J];
#pragma unroll
        for (int u = 0; u < R; u++)
#pragma unroll
          for (int j = 0; j < J; j++) {
            v[u][j] = u16x8{0, 0, 0, 0, 0, 0, 0, 0};
            if (J == 1 || act[j])
              v[u][j] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(p + u * step) + (int64_t)j * TX);
          }
#pragma unroll
        for (int u = 0; u < R; u++)
#pragma unroll
          for (int j = 0; j < J; j++) {
            float f[8];
            widen8<T>(v[u][j], f);
#pragma unroll
            for (int i = 0; i < 8; i++) m[j][i] = fmaxf(m[j][i], fabsf(f[i]));
          }
      };
      for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, p += U * step)
        do_rows(std::integral_constant<int, U>{});
      for (; row < it.row1; row += it.TY, p += step) do_rows(std::integral_constant<int, 1>{});
    } else {
      for (; row < it.row1; row += it.TY, p += step) m[0][0] = fmaxf(m[0][0], fabsf(widen<T>(*p)));
    }
  }
  if constexpr (J == 1) {
    if (it.TY > 1) {
#pragma unroll
      for (int i = 0; i < V; i++) red[i * kBlock + threadIdx.x] = m[0][i];
      __syncthreads();
      if (it.ty == 0) {
        for (int y = 1; y < it.TY; y++) {
#pragma unroll
          for (int i = 0; i < V; i++) m[0][i] = fmaxf(m[0][i], red[i * kBlock + y * TX + threadIdx.x]);
        }
      }
    }
  }
  // rchunks == 1: dst is the scale buffer and these are the final maxima; otherwise dst is the
  // workspace, [row chunk][batch * D] with chunk_stride = batch * D, and a second kernel finishes
  if (it.ty == 0) {
    const bool final_pass = rchunks == 1;
    const uint32_t rc = (blockIdx.x / ctiles) % rchunks;
#pragma unroll
    for (int j = 0; j < J; j++) {
      if (!act[j]) continue;
      float* out = dst + (int64_t)rc * chunk_stride + it.slab * D + (group0 + (int64_t)j * TX) * V;
      if (final_pass) {
#pragma unroll
        for (int i = 0; i < V; i++) out[i] = m[j][i] / 127.0f;
      } else if constexpr (V == 8) {
        reinterpret_cast<f32x4*>(out)[0] = f32x4{m[j][0], m[j][1], m[j][2], m[j][3]};
        reinterpret_cast<f32x4*>(out)[1] = f32x4{m[j][4], m[j][5], m[j][6], m[j][7]};
      } else {
#pragma unroll
        for (int i = 0; i < V; i++) out[i] = m[j][i];
      }
    }
  }
}

// ---- quantize --------------------------------------------------------------------------------
template <typename T, int V, int U>
__global__ __launch_bounds__(kMaxBlock) void quantize16_kernel(const uint16_t* __restrict__ x,
                                                               const float* __restrict__ scales,
                                                               int8_t* __restrict__ codes, int64_t N, int64_t D,
                                                               int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                               int64_t rows_per_chunk, int64_t groups,
                                                               int64_t x_slab, int64_t c_slab) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * V;
  float div[V];
  double rcp[V];
  if constexpr (V == 8) {
#pragma unroll
    for (int w = 0; w < 2; w++) {
      const f32x4 sv = *(reinterpret_cast<const f32x4*>(scales + it.slab * D + col) + w);
#pragma unroll
      for (int i = 0; i < 4; i++) {
        div[4 * w + i] = divisor_of(sv[i]);
        rcp[4 * w + i] = reciprocal_of(div[4 * w + i]);
      }
    }
  } else {
    rcp[0] = 0.0;
    const float s = scales[it.slab * D + col];
    div[0] = divisor_of(s);
  }
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  const uint16_t* px = x + it.slab * x_slab + row * D + col;  // slab pitches in elements
  int8_t* pc = codes + it.slab * c_slab + row * D + col;
  if constexpr (V == 8) {
    auto do_rows = [&](auto tag) {
      constexpr int R = decltype(tag)::value;
      u16x8 v[R];
#pragma unroll
      for (int u = 0; u < R; u++) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u16x8*>(px + u * step));
#pragma unroll
      for (int u = 0; u < R; u++) {
        float f[8];
        widen8<T>(v[u], f);
        u32x2 c;
#pragma unroll
        for (int w = 0; w < 2; w++) {
          uint32_t word = 0;
#pragma unroll
          for (int b = 0; b < 4; b++) word |= code_byte_r(f[4 * w + b], rcp[4 * w + b]) << (8 * b);
          c[w] = word;
        }
        __builtin_nontemporal_store(c, reinterpret_cast<u32x2*>(pc + u * step));
      }
    };
    for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * step)
      do_rows(std::integral_constant<int, U>{});
    for (; row < it.row1; row += it.TY, px += step, pc += step) do_rows(std::integral_constant<int, 1>{});
  } else {
    for (; row < it.row1; row += it.TY, px += step, pc += step) *pc = (int8_t)code_byte(widen<T>(*px), div[0]);
  }
}

// ---- dequantize --------------------------------------------------------------------------------
template <typename T, int V, int U>
__global__ __launch_bounds__(kMaxBlock) void dequantize16_kernel(const int8_t* __restrict__ codes,
                                                                 const float* __restrict__ scales,
                                                                 uint16_t* __restrict__ x_hat, int64_t N, int64_t D,
                                                                 int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                                 int64_t rows_per_chunk, int64_t groups) {
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  if (it.group >= groups) return;
  const int64_t col = it.group * V;
  float s[V];
  if constexpr (V == 8) {
#pragma unroll
    for (int w = 0; w < 2; w++) {
      const f32x4 sv = *(reinterpret_cast<const f32x4*>(scales + it.slab * D + col) + w);
#pragma unroll
      for (int i = 0; i < 4; i++) s[4 * w + i] = sv[i];
    }
  } else {
    s[0] = scales[it.slab * D + col];
  }
  const int64_t step = (int64_t)it.TY * D;
  int64_t row = it.row0 + it.ty;
  const int8_t* pc = codes + (it.slab * N + row) * D + col;
  uint16_t* px = x_hat + (it.slab * N + row) * D + col;
  if constexpr (V == 8) {
    auto do_rows = [&](auto tag) {
      constexpr int R = decltype(tag)::value;
      u32x2 c[R];
#pragma unroll
      // codes without the streaming hint, as in dequantize_kernel: they may stay in the memory-side cache
      for (int u = 0; u < R; u++) c[u] = *reinterpret_cast<const u32x2*>(pc + u * step);
#pragma unroll
      for (int u = 0; u < R; u++) {
        u16x8 o;
#pragma unroll
        for (int w = 0; w < 2; w++)
#pragma unroll
          for (int b = 0; b < 4; b++) {
            const int q = (int)(c[u][w] << (24 - 8 * b)) >> 24;
            o[4 * w + b] = narrow<T>((float)q * s[4 * w + b]);
          }
        __builtin_nontemporal_store(o, reinterpret_cast<u16x8*>(px + u * step));
      }
    };
    for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * step)
      do_rows(std::integral_constant<int, U>{});
    for (; row < it.row1; row += it.TY, px += step, pc += step) do_rows(std::integral_constant<int, 1>{});
  } else {
    for (; row < it.row1; row += it.TY, px += step, pc += step) *px = narrow<T>((float)(*pc) * s[0]);
  }
}

// ---- launchers ---------------------------------------------------------------------------------
// Default launch shapes of the 16-bit codec kernels, from a sweep over threads per workgroup
// (64..512), rows in flight per lane (1, 2, 4) and passes per workgroup (1, 2, 4) on [131072 x 8192]
// and [2048 x 4096 x 128]: single-wavefront workgroups with one row in flight that make a few passes
// beat the fp32 kernels' shapes here by 6-11 % (bf16 quantize 5.56 -> 5.91 / 6.05 TB/s, dequantize
// 5.79 -> 6.45 / 6.51 TB/s).
constexpr int kQ16Unroll = 1, kQ16Block = 64, kQ16Passes = 4, kD16Unroll = 1, kD16Block = 64, kD16Passes = 2;
template <typename T>
static kvq_status absmax16(const uint16_t* x, float* scales, int64_t batch, int64_t N, int64_t D,
                           hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  const Options& o = options();
  const int V = (D % 8 == 0 && aligned(x, 16)) ? 8 : 1;
  int J = 1;
  if (V == 8) {
    const int64_t groups = D / 8;
    // as in the fp32 reduction: workgroups that span whole rows wherever rows are that wide
    while (J < 4 && J < o.absmax_span && (int64_t)kBlock * J < groups) J *= 2;
  }
  constexpr int U1 = 8, UJ = 2;
  const int U = J == 1 ? U1 : UJ;
  // narrow rows: four workgroups per compute unit hide the conversion work behind each other's loads
  const int bpc = (J == 1 ? 4 : 1) * o.absmax_blocks_per_cu;
  Tiling t = make_tiling(batch, N, D, V * J, U, (int64_t)dev.cus * bpc, kBlock, 0);
  if (J > 1) {
    t.tx_log2 = 8;
    t.groups = D / V;
    t.ctiles = (uint32_t)((t.groups + (int64_t)kBlock * J - 1) / ((int64_t)kBlock * J));
    t.items = batch * (int64_t)t.rchunks * t.ctiles;
  }
  if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
  const int64_t total = batch * D;
  limit_row_chunks(&t, batch, N, absmax_chunk_cap(total));
  float* dst = scales;
  if (t.rchunks > 1) {
    Workspace ws;
    if (kvq_status s = get_workspace(stream, &ws)) return s;
    dst = ws.colmax;
  }
  const dim3 grid((uint32_t)t.items), block(kBlock);
#define KVQ_AM16(V_, J_, U_)                                                                                  \
  hipLaunchKernelGGL((absmax16_kernel<T, V_, J_, U_>), grid, block, 0, stream, x, dst, total, N, D, t.tx_log2, \
                     t.ctiles, t.rchunks, t.rows_per_chunk, t.groups)
  if (V == 1) KVQ_AM16(1, 1, U1);
  else if (J == 1) KVQ_AM16(8, 1, U1);
  else if (J == 2) KVQ_AM16(8, 2, UJ);
  else KVQ_AM16(8, 4, UJ);
#undef KVQ_AM16
  KVQ_HIP(hipGetLastError());
  if (t.rchunks > 1) return launch_absmax_finalize(dst, scales, total, t.rchunks, 127.0f, stream);
  return KVQ_OK;
}

template <typename T>
static kvq_status quantize16(const uint16_t* x, const float* scales, int8_t* codes, int64_t batch, int64_t N,
                             int64_t D, int64_t x_slab, int64_t c_slab, hipStream_t stream) {
  // both slab pitches are multiples of D, so the alignment of row 0 of slab 0 decides for all rows
  const bool vec = D % 8 == 0 && aligned(x, 16) && aligned(codes, 8) && aligned(scales, 16);
  int U;
  Tiling t;
  if (kvq_status s = stream_tiling(batch, N, D, vec ? 8 : 1, vec, kQ16Unroll, kQ16Block, &U, &t, kQ16Passes)) return s;
  const dim3 grid((uint32_t)t.items), block(t.block);
#define KVQ_Q16(U_) hipLaunchKernelGGL((quantize16_kernel<T, 8, U_>), grid, block, 0, stream, x, scales, codes, N, D, t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, x_slab, c_slab)
  if (!vec)
    hipLaunchKernelGGL((quantize16_kernel<T, 1, 1>), grid, block, 0, stream, x, scales, codes, N, D, t.tx_log2,
                       t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, x_slab, c_slab);
  else if (U == 1) KVQ_Q16(1);
  else if (U == 2) KVQ_Q16(2);
  else KVQ_Q16(4);
#undef KVQ_Q16
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

template <typename T>
static kvq_status dequantize16(const int8_t* codes, const float* scales, uint16_t* x_hat, int64_t batch, int64_t N,
                               int64_t D, hipStream_t stream) {
  const bool vec = D % 8 == 0 && aligned(x_hat, 16) && aligned(codes, 8) && aligned(scales, 16);
  int U;
  Tiling t;
  if (kvq_status s = stream_tiling(batch, N, D, vec ? 8 : 1, vec, kD16Unroll, kD16Block, &U, &t, kD16Passes)) return s;
  const dim3 grid((uint32_t)t.items), block(t.block);
#define KVQ_D16(U_) hipLaunchKernelGGL((dequantize16_kernel<T, 8, U_>), grid, block, 0, stream, codes, scales, x_hat, N, D, t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups)
  if (!vec)
    hipLaunchKernelGGL((dequantize16_kernel<T, 1, 1>), grid, block, 0, stream, codes, scales, x_hat, N, D,
                       t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
  else if (U == 1) KVQ_D16(1);
  else if (U == 2) KVQ_D16(2);
  else KVQ_D16(4);
#undef KVQ_D16
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

kvq_status launch_absmax_scales_16(int dtype, const void* x, float* scales, int64_t batch, int64_t N, int64_t D,
                                   hipStream_t stream) {
  const uint16_t* p = static_cast<const uint16_t*>(x);
  return dtype == KVQ_DTYPE_F16 ? absmax16<f16_tag>(p, scales, batch, N, D, stream)
                                : absmax16<bf16_tag>(p, scales, batch, N, D, stream);
}
kvq_status launch_quantize_16(int dtype, const void* x, const float* scales, int8_t* codes, int64_t batch,
                              int64_t N, int64_t D, hipStream_t stream) {
  return launch_quantize_16_strided(dtype, x, scales, codes, batch, N, D, N * D, N * D, stream);
}
kvq_status launch_quantize_16_strided(int dtype, const void* x, const float* scales, int8_t* codes, int64_t batch,
                                      int64_t N, int64_t D, int64_t x_slab, int64_t c_slab, hipStream_t stream) {
  const uint16_t* p = static_cast<const uint16_t*>(x);
  return dtype == KVQ_DTYPE_F16 ? quantize16<f16_tag>(p, scales, codes, batch, N, D, x_slab, c_slab, stream)
                                : quantize16<bf16_tag>(p, scales, codes, batch, N, D, x_slab, c_slab, stream);
}
kvq_status launch_dequantize_16(int dtype, const int8_t* codes, const float* scales, void* x_hat, int64_t batch,
                                int64_t N, int64_t D, hipStream_t stream) {
  uint16_t* p = static_cast<uint16_t*>(x_hat);
  return dtype == KVQ_DTYPE_F16 ? dequantize16<f16_tag>(codes, scales, p, batch, N, D, stream)
                                : dequantize16<bf16_tag>(codes, scales, p, batch, N, D, stream);
}

}  // namespace kvq
