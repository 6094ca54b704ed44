// Ablation points: the four work mappings the paper compares ("GPU Kernel Variants": naive, tiled,
// coarsened, vectorized) as gfx950 kernels, so that its qualitative findings (staging scales in shared
// memory buys nothing; wider memory operations are what helps) can be re-measured on CDNA4 next to the
// production kernel.  Only the mappings are the paper's -- one lane per element / the workgroup's scales
// staged in LDS / one lane per channel walking down the tokens / four adjacent channels per lane.  The
// kernels are this library's: one kernel over the library's work-item decomposition (a 1-D grid decoded
// into slab, row chunk and column tile, 64-bit indices, any shape), with the production arithmetic (IEEE
// divide, clamp, round-half-to-even, zero-scale guard), so all five designs produce identical codes.
// Launch shapes the paper does not state: workgroups are 64 lanes along a row x 4 rows (one wavefront per
// row); the coarsened design gets row chunks that give about 16 workgroups per compute unit.
#include <limits.h>

#include "kvq_internal.h"

namespace kvq {

constexpr int kAbTxLog2 = 6, kAbBlock = 256;  // 64 x 4 lanes
enum AbMode { kAbNaive, kAbTiled, kAbCoarsened, kAbVectorized };

__device__ __forceinline__ uint32_t ab_code(float x, float s) {
  float y = x / divisor_of(s);
  y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
  return __float_as_uint(y + kRoundMagic) & 0xffu;
}

template <int MODE>
__global__ __launch_bounds__(kAbBlock) void ablation_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ scales,
                                                            int8_t* __restrict__ codes, int64_t N, int64_t D,
                                                            uint32_t ctiles, uint32_t rchunks, int64_t rows_per_chunk,
                                                            int64_t groups) {
  constexpr int V = MODE == kAbVectorized ? 4 : 1;
  __shared__ float staged[1 << kAbTxLog2];
  const Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, kAbTxLog2);
  const bool active = it.group < groups;
  const int64_t col = it.group * V;
  const float* sp = scales + it.slab * D + col;
  if constexpr (MODE == kAbTiled) {
    // the lanes of the workgroup's first row fetch the tile's scales once; every row then reads them from LDS
    if (it.ty == 0 && active) staged[threadIdx.x] = *sp;
    __syncthreads();
  }
  if (!active) return;
  float kept = 0.0f;
  if constexpr (MODE == kAbCoarsened) kept = *sp;  // in a register for the whole walk
  for (int64_t row = it.row0 + it.ty; row < it.row1; row += it.TY) {
    const int64_t i = (it.slab * N + row) * D + col;
    if constexpr (MODE == kAbVectorized) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(x + i);
      const f32x4 s = *reinterpret_cast<const f32x4*>(sp);  // fetched again for every element, as in the design
      uint32_t w = 0;
#pragma unroll
      for (int k = 0; k < 4; k++) w |= ab_code(v[k], s[k]) << (8 * k);
      *reinterpret_cast<uint32_t*>(codes + i) = w;
    } else {
      float s;
      if constexpr (MODE == kAbNaive) s = *sp;
      else if constexpr (MODE == kAbTiled) s = staged[threadIdx.x & ((1 << kAbTxLog2) - 1)];
      else s = kept;
      codes[i] = (int8_t)ab_code(x[i], s);
    }
  }
}

kvq_status launch_quantize_variant(int variant, const float* x, const float* scales, int8_t* codes,
                                   int64_t batch, int64_t N, int64_t D, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  if (variant == KVQ_VARIANT_VECTORIZED && (D % 4 || !aligned(x, 16) || !aligned(scales, 16) || !aligned(codes, 4)))
    return KVQ_ERR_ARG;
  const int V = variant == KVQ_VARIANT_VECTORIZED ? 4 : 1;
  const int64_t TX = (int64_t)1 << kAbTxLog2, TY = kAbBlock / TX;
  const int64_t groups = (D + V - 1) / V;
  const int64_t ctiles = (groups + TX - 1) / TX;
  // one row per lane, except for the coarsened design, whose lanes walk a long row chunk
  int64_t rows = TY;
  if (variant == KVQ_VARIANT_COARSENED) {
    int64_t walkers = ((int64_t)dev.cus * 16 + ctiles * batch - 1) / (ctiles * batch);
    if (walkers < 1) walkers = 1;
    rows = (N + walkers - 1) / walkers;
    rows = (rows + TY - 1) / TY * TY;
  }
  const int64_t rchunks = (N + rows - 1) / rows;
  if (ctiles > INT32_MAX || rchunks > INT32_MAX || batch > INT32_MAX / ctiles ||
      batch * ctiles > INT32_MAX / rchunks)
    return KVQ_ERR_OVERFLOW;
  const dim3 grid((uint32_t)(batch * rchunks * ctiles)), block(kAbBlock);
#define KVQ_AB(MODE_)                                                                                        \
  hipLaunchKernelGGL((ablation_kernel<MODE_>), grid, block, 0, stream, x, scales, codes, N, D, (uint32_t)ctiles, \
                     (uint32_t)rchunks, rows, groups)
  if (variant == KVQ_VARIANT_NAIVE) KVQ_AB(kAbNaive);
  else if (variant == KVQ_VARIANT_TILED) KVQ_AB(kAbTiled);
  else if (variant == KVQ_VARIANT_COARSENED) KVQ_AB(kAbCoarsened);
  else KVQ_AB(kAbVectorized);
#undef KVQ_AB
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
