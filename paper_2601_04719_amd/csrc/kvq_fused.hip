// Scale computation and quantization of a small slab in one pass
// (paper: Eq. (scale_compute) + Eq. (quant_op); same results as the two separate kernels).
//
// When a whole [N x D] slab fits in the registers of one workgroup (at most 64 Ki elements: 1024
// lanes x 16 rows x 4 channels), the workgroup loads it once, reduces the column maxima through LDS,
// derives the scales, and quantizes straight from registers: x is read from HBM once instead of
// twice, and one launch replaces four.  Larger slabs cannot be done this way -- the first code of a
// column depends on its last row -- and take the two-pass path.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

constexpr int kFusedBlock = 1024;
constexpr int kFusedMaxRows = 16;  // rows per lane


template <int R>
__global__ __launch_bounds__(kFusedBlock) void fused_slab_kernel(const float* __restrict__ x,
                                                                 float* __restrict__ scales,
                                                                 int8_t* __restrict__ codes, int64_t N, int64_t D,
                                                                 int tx_log2) {
  __shared__ float red[4][kFusedBlock];
  const int tid = threadIdx.x;
  const int TX = 1 << tx_log2, TY = (int)blockDim.x >> tx_log2;
  const int tx = tid & (TX - 1), ty = tid >> tx_log2;
  const int64_t slab = blockIdx.x;
  const bool active = (int64_t)tx * 4 < D;
  const float* xs = x + slab * N * D + (int64_t)tx * 4;
  int8_t* cs = codes + slab * N * D + (int64_t)tx * 4;

  f32x4 v[R];
  float m[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int u = 0; u < R; u++) {
    const int64_t row = ty + (int64_t)u * TY;
    v[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (active && row < N) v[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(xs + row * D));
  }
#pragma unroll
  for (int u = 0; u < R; u++)
#pragma unroll
    for (int i = 0; i < 4; i++) m[i] = fmaxf(m[i], fabsf(v[u][i]));

  // column maxima over the TY lanes that share a column group: tree in LDS, result in row ty == 0
#pragma unroll
  for (int i = 0; i < 4; i++) red[i][tid] = m[i];
  __syncthreads();
  for (int s = TY >> 1; s > 0; s >>= 1) {
    if (ty < s) {
#pragma unroll
      for (int i = 0; i < 4; i++) red[i][tid] = fmaxf(red[i][tid], red[i][tid + s * TX]);
    }
    __syncthreads();
  }
  f32x4 sc;
  float div[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    sc[i] = red[i][tx] / 127.0f;                           // the one IEEE divide per channel
    div[i] = divisor_of(sc[i]);
  }
  if (active && ty == 0) *reinterpret_cast<f32x4*>(scales + slab * D + (int64_t)tx * 4) = sc;

#pragma unroll
  for (int u = 0; u < R; u++) {
    const int64_t row = ty + (int64_t)u * TY;
    if (active && row < N) {
      uint32_t w = 0;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        float y = v[u][i] / div[i];
        y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
        w |= (__float_as_uint(y + kRoundMagic) & 0xffu) << (8 * i);
      }
      __builtin_nontemporal_store(w, reinterpret_cast<uint32_t*>(cs + row * D));
    }
  }
}

static int ceil_log2_int(int64_t v) {
  int l = 0;
  while (((int64_t)1 << l) < v) l++;
  return l;
}

bool fused_slab_applicable(const float* x, const float* scales, const int8_t* codes, int64_t N, int64_t D) {
  if (D % 4 || !aligned(x, 16) || !aligned(scales, 16) || !aligned(codes, 4)) return false;
  const int64_t groups = D / 4;
  if (groups > kFusedBlock) return false;
  const int64_t TX = (int64_t)1 << ceil_log2_int(groups);
  const int64_t TY = kFusedBlock / TX;
  return (N + TY - 1) / TY <= kFusedMaxRows;
}

kvq_status launch_fused_slab(const float* x, float* scales, int8_t* codes, int64_t batch, int64_t N, int64_t D,
                             hipStream_t stream) {
  if (batch > INT32_MAX) return KVQ_ERR_OVERFLOW;
  const int64_t groups = D / 4;
  const int tx_log2 = ceil_log2_int(groups);
  const int64_t TX = (int64_t)1 << tx_log2;
  // a small slab does not need all 1024 lanes: shrink the workgroup while 1 row per lane still covers it
  int block = kFusedBlock;
  while (block > 64 && block / 2 >= TX && (N + (block / 2) / TX - 1) / ((block / 2) / TX) <= 1) block /= 2;
  const int64_t TY = block / TX;
  const int64_t rows = (N + TY - 1) / TY;
  const dim3 grid((uint32_t)batch), blk(block);
#define KVQ_FUSED(R_) \
  hipLaunchKernelGGL((fused_slab_kernel<R_>), grid, blk, 0, stream, x, scales, codes, N, D, tx_log2)
  if (rows <= 1) KVQ_FUSED(1);
  else if (rows <= 2) KVQ_FUSED(2);
  else if (rows <= 4) KVQ_FUSED(4);
  else if (rows <= 8) KVQ_FUSED(8);
  else KVQ_FUSED(16);
#undef KVQ_FUSED
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
