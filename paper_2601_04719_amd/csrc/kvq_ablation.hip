// Ablation points: gfx950 renditions of the four kernel designs the paper compares
// ("GPU Kernel Variants": naive, tiled, coarsened, vectorized), so that its qualitative findings
// (staging scales in shared memory buys nothing; wider memory operations are what helps) can be
// re-measured on CDNA4 next to the production kernel.  They are written from the paper's
// descriptions of the four work mappings; the arithmetic is the production one (IEEE divide, clamp,
// round-half-to-even, zero-scale guard), so all five produce identical codes.  Launch shapes the
// paper does not state: workgroups are 64 channels x 4 tokens (one wavefront per token row); the
// coarsened design walks tokens with as many grid rows as give about 16 workgroups per compute unit.
#include "kvq_internal.h"

namespace kvq {

constexpr int kAbX = 64, kAbY = 4;

__device__ __forceinline__ int8_t ab_code(float x, float s) {
  const float d = divisor_of(s);
  float y = x / d;
  y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
  return (int8_t)(__float_as_uint(y + kRoundMagic) & 0xffu);
}

// "naive": one lane per element; every lane fetches its own scale.
__global__ __launch_bounds__(kAbX* kAbY) void ab_naive(const float* __restrict__ x, const float* __restrict__ scales,
                                                      int8_t* __restrict__ codes, int64_t N, int64_t D,
                                                      uint32_t row_blocks) {
  const int64_t slab = blockIdx.y / row_blocks;
  const int64_t t = (int64_t)(blockIdx.y % row_blocks) * kAbY + threadIdx.y;
  const int64_t d = (int64_t)blockIdx.x * kAbX + threadIdx.x;
  if (t < N && d < D) {
    const int64_t i = (slab * N + t) * D + d;
    codes[i] = ab_code(x[i], scales[slab * D + d]);
  }
}

// "tiled": the workgroup's 64 scales are staged in LDS by its first token row, then shared.
__global__ __launch_bounds__(kAbX* kAbY) void ab_tiled(const float* __restrict__ x, const float* __restrict__ scales,
                                                      int8_t* __restrict__ codes, int64_t N, int64_t D,
                                                      uint32_t row_blocks) {
  __shared__ float s_tile[kAbX];
  const int64_t slab = blockIdx.y / row_blocks;
  const int64_t t = (int64_t)(blockIdx.y % row_blocks) * kAbY + threadIdx.y;
  const int64_t d = (int64_t)blockIdx.x * kAbX + threadIdx.x;
  if (threadIdx.y == 0 && d < D) s_tile[threadIdx.x] = scales[slab * D + d];
  __syncthreads();
  if (t < N && d < D) {
    const int64_t i = (slab * N + t) * D + d;
    codes[i] = ab_code(x[i], s_tile[threadIdx.x]);
  }
}

// "coarsened": one lane per channel keeps its scale in a register and walks down the tokens,
// gridDim.y workgroup rows apart.
__global__ __launch_bounds__(kAbX* kAbY) void ab_coarsened(const float* __restrict__ x,
                                                          const float* __restrict__ scales,
                                                          int8_t* __restrict__ codes, int64_t N, int64_t D,
                                                          uint32_t walkers) {
  const int64_t slab = blockIdx.y / walkers;
  const int64_t d = (int64_t)blockIdx.x * kAbX + threadIdx.x;
  if (d >= D) return;
  const float s = scales[slab * D + d];
  const int64_t stride = (int64_t)walkers * kAbY;
  for (int64_t t = (int64_t)(blockIdx.y % walkers) * kAbY + threadIdx.y; t < N; t += stride) {
    const int64_t i = (slab * N + t) * D + d;
    codes[i] = ab_code(x[i], s);
  }
}

// "vectorized": four adjacent channels per lane: one 16-byte load of x and of the scales, one
// 4-byte store of codes.  Needs D % 4 == 0 and 16-byte aligned rows.
__global__ __launch_bounds__(kAbX* kAbY) void ab_vectorized(const float* __restrict__ x,
                                                           const float* __restrict__ scales,
                                                           int8_t* __restrict__ codes, int64_t N, int64_t D,
                                                           uint32_t row_blocks) {
  const int64_t slab = blockIdx.y / row_blocks;
  const int64_t t = (int64_t)(blockIdx.y % row_blocks) * kAbY + threadIdx.y;
  const int64_t d = ((int64_t)blockIdx.x * kAbX + threadIdx.x) * 4;
  if (t < N && d < D) {
    const int64_t i = (slab * N + t) * D + d;
    const f32x4 v = *reinterpret_cast<const f32x4*>(x + i);
    const f32x4 s = *reinterpret_cast<const f32x4*>(scales + slab * D + d);
    uint32_t w = 0;
#pragma unroll
    for (int k = 0; k < 4; k++) w |= (uint32_t)(uint8_t)ab_code(v[k], s[k]) << (8 * k);
    *reinterpret_cast<uint32_t*>(codes + i) = w;
  }
}

kvq_status launch_quantize_variant(int variant, const float* x, const float* scales, int8_t* codes,
                                   int64_t batch, int64_t N, int64_t D, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  const dim3 block(kAbX, kAbY);
  const int64_t row_blocks = (N + kAbY - 1) / kAbY;
  const int64_t lanes_x = variant == KVQ_VARIANT_VECTORIZED ? D / 4 : D;
  const int64_t gx = (lanes_x + kAbX - 1) / kAbX;
  if (gx > INT32_MAX) return KVQ_ERR_OVERFLOW;
  if (variant == KVQ_VARIANT_COARSENED) {
    int64_t walkers = ((int64_t)dev.cus * 16 + gx * batch - 1) / (gx * batch);
    if (walkers < 1) walkers = 1;
    if (walkers > row_blocks) walkers = row_blocks;
    if (batch * walkers > 65535) return KVQ_ERR_OVERFLOW;
    hipLaunchKernelGGL(ab_coarsened, dim3((uint32_t)gx, (uint32_t)(batch * walkers)), block, 0, stream, x, scales,
                       codes, N, D, (uint32_t)walkers);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
  }
  // the 2-D designs put (slab, token block) on grid.y, which holds at most 65535 rows: larger problems
  // are issued as several launches over row ranges
  if (variant == KVQ_VARIANT_VECTORIZED && (D % 4 || !aligned(x, 16) || !aligned(scales, 16) || !aligned(codes, 4)))
    return KVQ_ERR_ARG;
  const int64_t max_rows_per_launch = (int64_t)65535 * kAbY;
  for (int64_t b = 0; b < batch; b++) {
    for (int64_t r0 = 0; r0 < N; r0 += max_rows_per_launch) {
      const int64_t n = N - r0 < max_rows_per_launch ? N - r0 : max_rows_per_launch;
      const uint32_t rb = (uint32_t)((n + kAbY - 1) / kAbY);
      const float* xp = x + (b * N + r0) * D;
      int8_t* cp = codes + (b * N + r0) * D;
      const float* sp = scales + b * D;
      const dim3 grid((uint32_t)gx, rb);
      if (variant == KVQ_VARIANT_NAIVE) hipLaunchKernelGGL(ab_naive, grid, block, 0, stream, xp, sp, cp, n, D, rb);
      else if (variant == KVQ_VARIANT_TILED) hipLaunchKernelGGL(ab_tiled, grid, block, 0, stream, xp, sp, cp, n, D, rb);
      else hipLaunchKernelGGL(ab_vectorized, grid, block, 0, stream, xp, sp, cp, n, D, rb);
      KVQ_HIP(hipGetLastError());
    }
  }
  return KVQ_OK;
}

}  // namespace kvq
