// Scale computation: scales[b,d] = max_t |x[b,t,d]| / 127
// (paper: Eq. (scale), Eq. (scale_compute), Algorithm "Compute Scales").
//
// The paper computes scales on the host only.  Here the column maximum is a
// streaming reduction over rows: every lane owns V adjacent channels, reads
// its rows with 16-byte loads that a wavefront issues as whole contiguous row
// segments, keeps V running maxima in registers, and at the end the maxima of
// the lanes that share channels are combined in LDS and merged across
// workgroups with an atomic max on the bit pattern of the (non-negative)
// float, whose unsigned order equals the float order.  max is associative and
// commutative, so the result does not depend on the launch shape.
//
// Unlike the codec kernels, workgroups here walk long row chunks (about eight
// workgroups per compute unit): one-shot workgroups of a few rows, each ending
// in a device-scope read and an atomic per channel, measured 1.5x slower.
#include "kvq_internal.h"

namespace kvq {

__global__ __launch_bounds__(kBlock) void fill_zero_u32(uint32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// One IEEE fp32 divide per channel, in place over the max bit patterns.
__global__ __launch_bounds__(kBlock) void finalize_scales(float* scales, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) scales[i] = scales[i] / 127.0f;
}

// |v| joins the running maximum only when strictly larger, as in the algorithm;
// fmaxf(m, |v|) is the same function on finite data.
__device__ __forceinline__ float absmax_step(float m, float v) { return fmaxf(m, fabsf(v)); }

template <int V, int U, bool NT>
__global__ __launch_bounds__(kBlock) void absmax_kernel(const float* __restrict__ x,
                                                        uint32_t* __restrict__ max_bits, int64_t N, int64_t D,
                                                        int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                        int64_t rows_per_chunk, int64_t groups) {
  __shared__ float red[kBlock * V];
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  const bool active = it.group < groups;
  float m[V];
#pragma unroll
  for (int i = 0; i < V; i++) m[i] = 0.0f;

  if (active) {
    const float* base = x + (it.slab * N) * D + it.group * V;
    const int64_t step = (int64_t)it.TY * D;  // elements between successive rows of this lane
    int64_t row = it.row0 + it.ty;
    const float* p = base + row * D;
    if constexpr (V == 4) {
      // main loop: U rows in flight
      for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, p += U * step) {
        f32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; u++) v[u] = ld<NT>(reinterpret_cast<const f32x4*>(p + u * step));
#pragma unroll
        for (int u = 0; u < U; u++) {
          m[0] = absmax_step(m[0], v[u].x);
          m[1] = absmax_step(m[1], v[u].y);
          m[2] = absmax_step(m[2], v[u].z);
          m[3] = absmax_step(m[3], v[u].w);
        }
      }
      for (; row < it.row1; row += it.TY, p += step) {
        const f32x4 v = ld<NT>(reinterpret_cast<const f32x4*>(p));
        m[0] = absmax_step(m[0], v.x);
        m[1] = absmax_step(m[1], v.y);
        m[2] = absmax_step(m[2], v.z);
        m[3] = absmax_step(m[3], v.w);
      }
    } else {
      static_assert(V == 1, "absmax lanes are 4-wide or scalar");
      for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, p += U * step) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; u++) v[u] = p[u * step];
#pragma unroll
        for (int u = 0; u < U; u++) m[0] = absmax_step(m[0], v[u]);
      }
      for (; row < it.row1; row += it.TY, p += step) m[0] = absmax_step(m[0], *p);
    }
  }

  // combine the TY lanes that share a channel group (LDS), then one atomic per channel
  if (it.TY > 1) {
#pragma unroll
    for (int i = 0; i < V; i++) red[i * kBlock + threadIdx.x] = m[i];
    __syncthreads();
    if (it.ty == 0) {
      const int TX = 1 << tx_log2;
      for (int y = 1; y < it.TY; y++) {
#pragma unroll
        for (int i = 0; i < V; i++) m[i] = fmaxf(m[i], red[i * kBlock + y * TX + threadIdx.x]);
      }
    }
  }
  if (active && it.ty == 0) {
    uint32_t* out = max_bits + it.slab * D + it.group * V;
#pragma unroll
    for (int i = 0; i < V; i++) {
      const uint32_t bits = __float_as_uint(m[i]);
      if (bits != 0u) atomicMax(out + i, bits);
    }
  }
}

template <int V, int U>
static kvq_status launch_absmax_t(const float* x, uint32_t* bits, int64_t N, int64_t D, const Tiling& t,
                                  bool nt, hipStream_t stream) {
  const dim3 grid((uint32_t)t.items), block(kBlock);
  if (nt)
    hipLaunchKernelGGL((absmax_kernel<V, U, true>), grid, block, 0, stream, x, bits, N, D, t.tx_log2, t.ctiles,
                       t.rchunks, t.rows_per_chunk, t.groups);
  else
    hipLaunchKernelGGL((absmax_kernel<V, U, false>), grid, block, 0, stream, x, bits, N, D, t.tx_log2,
                       t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

kvq_status launch_absmax_scales(const float* x, float* scales, int64_t batch, int64_t N, int64_t D,
                                hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  const Options& o = options();
  const int V = (D % 4 == 0 && aligned(x, 16)) ? 4 : 1;
  const int U = o.absmax_unroll;
  int passes = o.absmax_passes;
  Tiling t = make_tiling(batch, N, D, V, U, (int64_t)dev.cus * o.blocks_per_cu, kBlock, passes);
  while (t.items > ((int64_t)1 << 30) && passes > 0 && passes < (1 << 20)) {
    passes *= 2;
    t = make_tiling(batch, N, D, V, U, (int64_t)dev.cus * o.blocks_per_cu, kBlock, passes);
  }
  if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
  const int64_t n_scales = batch * D;
  const int64_t small_blocks = (n_scales + kBlock - 1) / kBlock;
  if (small_blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  uint32_t* bits = reinterpret_cast<uint32_t*>(scales);

  hipLaunchKernelGGL(fill_zero_u32, dim3((uint32_t)small_blocks), dim3(kBlock), 0, stream, bits, n_scales);
  KVQ_HIP(hipGetLastError());
  const bool nt = o.nontemporal != 0;
  kvq_status s;
  if (V == 4 && U == 4) s = launch_absmax_t<4, 4>(x, bits, N, D, t, nt, stream);
  else if (V == 4 && U == 8) s = launch_absmax_t<4, 8>(x, bits, N, D, t, nt, stream);
  else if (V == 4) s = launch_absmax_t<4, 16>(x, bits, N, D, t, nt, stream);
  else if (U == 4) s = launch_absmax_t<1, 4>(x, bits, N, D, t, false, stream);
  else if (U == 8) s = launch_absmax_t<1, 8>(x, bits, N, D, t, false, stream);
  else s = launch_absmax_t<1, 16>(x, bits, N, D, t, false, stream);
  if (s != KVQ_OK) return s;
  hipLaunchKernelGGL(finalize_scales, dim3((uint32_t)small_blocks), dim3(kBlock), 0, stream, scales, n_scales);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
