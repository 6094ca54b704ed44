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
// Unlike the codec kernels, workgroups here walk long row chunks: one workgroup
// per compute unit, each lane owning up to 8 column groups so that the workgroup
// reads whole rows -- one fat contiguous stream per compute unit.  Measured on
// the 1B-element shape: 7.0 TB/s, against 6.5 TB/s with eight 4 KiB-wide
// workgroups per compute unit, and 4 TB/s for one-shot workgroups of a few rows
// (each ending in an atomic per channel).
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

__global__ __launch_bounds__(kBlock) void fill_zero_u32(uint32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// One IEEE fp32 divide per channel, in place over the max bit patterns.
// qmax = 127 (8-bit codes) or 7 (4-bit codes).
__global__ __launch_bounds__(kBlock) void finalize_scales(float* scales, int64_t n, float qmax) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i < n) scales[i] = scales[i] / qmax;
}

// |v| joins the running maximum only when strictly larger, as in the algorithm;
// fmaxf(m, |v|) is the same function on finite data.
__device__ __forceinline__ float absmax_step(float m, float v) { return fmaxf(m, fabsf(v)); }

// A lane owns J groups of V adjacent channels, TX groups apart: with J * TX * V
// >= D a workgroup reads whole rows, i.e. one contiguous stream per workgroup.
template <int V, int J, int U, bool NT>
__global__ __launch_bounds__(kBlock) void absmax_kernel(const float* __restrict__ x,
                                                        uint32_t* __restrict__ max_bits, int64_t N, int64_t D,
                                                        int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                        int64_t rows_per_chunk, int64_t groups) {
  __shared__ float red[J == 1 ? kBlock * V : 1];
  // decode_item numbers column tiles in units of TX groups; a tile here is J of those
  Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  const int TX = 1 << tx_log2;
  const int64_t group0 = (it.group - (threadIdx.x & (TX - 1))) * J + (threadIdx.x & (TX - 1));
  float m[J][V];
#pragma unroll
  for (int j = 0; j < J; j++)
#pragma unroll
    for (int i = 0; i < V; i++) m[j][i] = 0.0f;
  bool act[J];
#pragma unroll
  for (int j = 0; j < J; j++) act[j] = group0 + (int64_t)j * TX < groups;

  if (act[0]) {
    const float* base = x + (it.slab * N) * D + group0 * V;
    const int64_t step = (int64_t)it.TY * D;  // elements between successive rows of this lane
    int64_t row = it.row0 + it.ty;
    const float* p = base + row * D;
    if constexpr (V == 4) {
      auto do_rows = [&](auto tag) {
        constexpr int R = decltype(tag)::value;
        f32x4 v[R][J];
#pragma unroll
        for (int u = 0; u < R; u++)
#pragma unroll
          for (int j = 0; j < J; j++)
            if (J == 1 || act[j]) v[u][j] = ld<NT>(reinterpret_cast<const f32x4*>(p + u * step) + (int64_t)j * TX);
            else v[u][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < R; u++)
#pragma unroll
          for (int j = 0; j < J; j++) {
            m[j][0] = absmax_step(m[j][0], v[u][j].x);
            m[j][1] = absmax_step(m[j][1], v[u][j].y);
            m[j][2] = absmax_step(m[j][2], v[u][j].z);
            m[j][3] = absmax_step(m[j][3], v[u][j].w);
          }
      };
      for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, p += U * step)
        do_rows(std::integral_constant<int, U>{});
      for (; row < it.row1; row += it.TY, p += step) do_rows(std::integral_constant<int, 1>{});
    } else {
      static_assert(V == 1 && J == 1, "absmax lanes are 4-wide or scalar");
      for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, p += U * step) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; u++) v[u] = p[u * step];
#pragma unroll
        for (int u = 0; u < U; u++) m[0][0] = absmax_step(m[0][0], v[u]);
      }
      for (; row < it.row1; row += it.TY, p += step) m[0][0] = absmax_step(m[0][0], *p);
    }
  }

  // combine the TY lanes that share a channel group (LDS; only rows narrower than a workgroup
  // have TY > 1, and those use J == 1), then one atomic per channel
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
  if (it.ty == 0) {
#pragma unroll
    for (int j = 0; j < J; j++) {
      if (!act[j]) continue;
      uint32_t* out = max_bits + it.slab * D + (group0 + (int64_t)j * TX) * V;
#pragma unroll
      for (int i = 0; i < V; i++) {
        const uint32_t bits = __float_as_uint(m[j][i]);
        if (bits != 0u) atomicMax(out + i, bits);
      }
    }
  }
}

template <int V, int J, int U>
static kvq_status launch_absmax_t(const float* x, uint32_t* bits, int64_t N, int64_t D, const Tiling& t,
                                  bool nt, hipStream_t stream) {
  const dim3 grid((uint32_t)t.items), block(kBlock);
  if (nt)
    hipLaunchKernelGGL((absmax_kernel<V, J, U, true>), grid, block, 0, stream, x, bits, N, D, t.tx_log2,
                       t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
  else
    hipLaunchKernelGGL((absmax_kernel<V, J, U, false>), grid, block, 0, stream, x, bits, N, D, t.tx_log2,
                       t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

kvq_status launch_absmax_scales(const float* x, float* scales, int64_t batch, int64_t N, int64_t D,
                                hipStream_t stream, float qmax) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  const Options& o = options();
  const int V = (D % 4 == 0 && aligned(x, 16)) ? 4 : 1;
  // J column groups per lane: as many as it takes for a workgroup to span whole rows, at most 8 --
  // but a wider workgroup means more row chunks for the same number of workgroups, and every chunk
  // ends in one atomic per channel.  Keep at least about 512 rows per workgroup: measured on
  // [16384 x 8192] J = 1 / 4 / 8 give 5.9 / 5.7 / 5.3 TB/s, on [4096 x 8192] 3.6 / 3.5 / 2.6, while
  // from [65536 x 8192] up the wide forms win (6.3 / 6.8 / 6.8; 7.0 for J = 8 at 131072 rows).
  int J = 1;
  if (V == 4) {
    const int64_t groups = D / 4;
    const int64_t elements = batch * N * D;
    const int64_t j_rows = elements / ((int64_t)dev.cus << 19);  // 512 rows x 1024 channels per unit of J
    while (J < o.absmax_span && J * 2 <= j_rows && (int64_t)kBlock * J < groups) J *= 2;
  }
  // rows in flight: J * U 16-byte loads per lane, at most 16
  int U = o.absmax_unroll;
  while (J * U > 16) U /= 2;
  if (J >= 2 && U > 4) U = 4;
  int passes = o.absmax_passes;
  // tiling in units of J * V channels per lane
  Tiling t = make_tiling(batch, N, D, V * J, U, (int64_t)dev.cus * o.absmax_blocks_per_cu, kBlock, passes);
  while (t.items > ((int64_t)1 << 30) && passes > 0 && passes < (1 << 20)) {
    passes *= 2;
    t = make_tiling(batch, N, D, V * J, U, (int64_t)dev.cus * o.absmax_blocks_per_cu, kBlock, passes);
  }
  if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
  if (J > 1) {
    // make_tiling sized TX for D / (V*J) lane-columns; with J > 1 rows are at least a workgroup wide
    t.tx_log2 = 8;
    t.groups = D / V;
    t.ctiles = (uint32_t)((t.groups + (int64_t)kBlock * J - 1) / ((int64_t)kBlock * J));
    t.items = batch * (int64_t)t.rchunks * t.ctiles;
  }
  const int64_t n_scales = batch * D;
  const int64_t small_blocks = (n_scales + kBlock - 1) / kBlock;
  if (small_blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  uint32_t* bits = reinterpret_cast<uint32_t*>(scales);

  hipLaunchKernelGGL(fill_zero_u32, dim3((uint32_t)small_blocks), dim3(kBlock), 0, stream, bits, n_scales);
  KVQ_HIP(hipGetLastError());
  const bool nt = o.nontemporal != 0;
  kvq_status s;
#define KVQ_AM(V_, J_, U_) s = launch_absmax_t<V_, J_, U_>(x, bits, N, D, t, nt, stream)
  if (V == 4 && J == 8 && U == 4) KVQ_AM(4, 8, 4);
  else if (V == 4 && J == 8) KVQ_AM(4, 8, 2);
  else if (V == 4 && J == 4 && U == 4) KVQ_AM(4, 4, 4);
  else if (V == 4 && J == 4) KVQ_AM(4, 4, 2);
  else if (V == 4 && J == 2 && U == 4) KVQ_AM(4, 2, 4);
  else if (V == 4 && J == 2) KVQ_AM(4, 2, 2);
  else if (V == 4 && U == 4) KVQ_AM(4, 1, 4);
  else if (V == 4 && U == 8) KVQ_AM(4, 1, 8);
  else if (V == 4) KVQ_AM(4, 1, 16);
  else if (U == 4) KVQ_AM(1, 1, 4);
  else if (U == 8) KVQ_AM(1, 1, 8);
  else KVQ_AM(1, 1, 16);
#undef KVQ_AM
  if (s != KVQ_OK) return s;
  hipLaunchKernelGGL(finalize_scales, dim3((uint32_t)small_blocks), dim3(kBlock), 0, stream, scales, n_scales, qmax);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
