// Scale computation and quantization in one pass
// (paper: Eq. (scale_compute) + Eq. (quant_op); same results as the two separate kernels).
//
// The first code of a column depends on the column's last row, so a single pass has to hold every
// row of the columns it works on.  Channels are independent, so the unit is a column tile: all N rows
// of TX groups of 4 adjacent channels, at most 64 Ki elements (1024 lanes x 16 rows x 4 channels),
// held in the registers of one workgroup.  The workgroup loads its tile once, reduces the column
// maxima through LDS, derives the scales, and quantizes straight from registers: x is read from HBM
// once instead of twice, and one launch replaces four.  A slab of up to 64 Ki elements is one tile;
// a taller slab is cut into tiles, by default no narrower than 32 channels (128-byte row segments of
// x, 32-byte segments of codes), which reaches N = 2048; narrower tiles are possible down to 16
// channels (N = 4096) but do not beat two passes (see fused_tile_tx_log2).  Neighbouring tiles share
// cache lines, so the tiles of a slab are numbered such that they run on the same XCD one after the
// other and meet in its L2.  Slabs of 2049 to 4096 rows have a kernel of their own (kvq_fused_tall.hip);
// taller ones take the two-pass path.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

constexpr int kFusedBlock = 1024;
constexpr int kFusedMaxRows = 16;  // rows per lane


constexpr int kXcds = 8;  // workgroup i of a launch is handed to XCD i % 8

// NT: streaming stores.  Tiles narrower than a cache line of codes (128 channels) store plainly instead,
// so that the pieces of a line written by neighbouring tiles can meet in L2 before it goes out.
template <int R, bool NT>
__global__ __launch_bounds__(kFusedBlock) void fused_slab_kernel(const float* __restrict__ x,
                                                                 float* __restrict__ scales,
                                                                 int8_t* __restrict__ codes, int64_t batch, int64_t N,
                                                                 int64_t D, int tx_log2, uint32_t ctiles) {
  __shared__ float red[4][kFusedBlock];
  const int tid = threadIdx.x;
  const int TX = 1 << tx_log2, TY = (int)blockDim.x >> tx_log2;
  const int tx = tid & (TX - 1), ty = tid >> tx_log2;
  // XCD i % 8 takes the slabs congruent to it, tile after tile: local index j -> slab j / ctiles, tile j % ctiles
  int64_t slab = blockIdx.x;
  uint32_t tile = 0;
  if (ctiles > 1) {
    const uint32_t xcd = blockIdx.x % kXcds, j = blockIdx.x / kXcds;
    slab = (int64_t)xcd + (int64_t)kXcds * (j / ctiles);
    tile = j % ctiles;
    if (slab >= batch) return;  // the last round of slabs may not fill all XCDs (uniform for the workgroup)
  }
  const int64_t col = ((int64_t)tile * TX + tx) * 4;
  const bool active = col < D;
  const float* xs = x + slab * N * D + col;
  int8_t* cs = codes + slab * N * D + col;

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
  double rcp[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    sc[i] = red[i][tx] / 127.0f;                           // the one IEEE divide per channel
    rcp[i] = reciprocal_of(divisor_of(sc[i]));
  }
  if (active && ty == 0) *reinterpret_cast<f32x4*>(scales + slab * D + col) = sc;

#pragma unroll
  for (int u = 0; u < R; u++) {
    const int64_t row = ty + (int64_t)u * TY;
    if (active && row < N) {
      uint32_t w = 0;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        float y = quotient_by(v[u][i], rcp[i]);  // the bits of v / divisor, without the divide sequence
        y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
        w |= (__float_as_uint(y + kRoundMagic) & 0xffu) << (8 * i);
      }
      st<NT>(reinterpret_cast<uint32_t*>(cs + row * D), w);
    }
  }
}

// Lanes along a row (a power of two, log2 returned) of the widest column tile that fits with at most
// `max_rows` rows per lane and at least `min_lanes` lanes along a row (unless the rows are narrower).  -1: none.
static int widest_tile_tx_log2(int64_t N, int64_t D, int max_rows, int64_t min_lanes) {
  const int64_t groups = D / 4;
  int best = -1;
  for (int l = 0; ((int64_t)1 << l) <= kFusedBlock; l++) {
    const int64_t TX = (int64_t)1 << l, TY = kFusedBlock / TX;
    if ((N + TY - 1) / TY > max_rows) break;   // wider tiles only have fewer lanes per column
    if (TX < min_lanes && TX < groups) continue;
    best = l;
    if (TX >= groups) break;                    // the whole row
  }
  return best;
}

// The tile shape of the single-pass form, or -1 if the slab is too tall for it.
//  - Rows per lane: 16 rows (64 data registers, 106 in all) leave room for one 1024-lane workgroup per
//    compute unit, whose load, reduce and store phases then run one after the other; 8 rows (58
//    registers) let two workgroups share the unit and overlap.  Measured, 8 against 16 rows per lane:
//    [512 x 1024 x 256] 0.137 against 0.168 ms, [4096 x 512 x 128] 0.260 against 0.294 ms -- so 8 rows
//    where that still gives tiles of the minimum width, else 16.
//  - Width: narrow tiles read and write short row segments.  With plain (cached) stores the pieces of a
//    code line written by neighbouring tiles mostly meet in L2 (with streaming stores a 4-lane tile
//    wrote 2.8 bytes per element instead of 1 and took 0.32 ms on [256 x 4096 x 128]); even so 4-lane
//    tiles only tie with two passes there (0.187 against 0.183 ms: 4.97 B fetched and 1.41 B written per
//    element), while 8-lane tiles win ([256 x 2048 x 256]: 0.163 against 0.182 ms).  Hence 8 lanes by default.
static int fused_tile_tx_log2(int64_t N, int64_t D, int* max_rows_out) {
  const Options& o = options();
  const int candidates[2] = {8, kFusedMaxRows};
  for (int c = 0; c < 2; c++) {
    const int rows = o.fused_max_rows > 0 ? o.fused_max_rows : candidates[c];
    const int l = widest_tile_tx_log2(N, D, rows, o.fused_min_lanes);
    if (l >= 0) {
      if (max_rows_out) *max_rows_out = rows;
      return l;
    }
    if (o.fused_max_rows > 0) break;
  }
  return -1;
}

bool fused_slab_applicable(const float* x, const float* scales, const int8_t* codes, int64_t N, int64_t D) {
  if (D % 4 || !aligned(x, 16) || !aligned(scales, 16) || !aligned(codes, 4)) return false;
  return fused_tile_tx_log2(N, D, nullptr) >= 0;
}

kvq_status launch_fused_slab(const float* x, float* scales, int8_t* codes, int64_t batch, int64_t N, int64_t D,
                             hipStream_t stream) {
  const int64_t groups = D / 4;
  int max_rows = kFusedMaxRows;
  const int tx_log2 = fused_tile_tx_log2(N, D, &max_rows);
  if (tx_log2 < 0) return KVQ_ERR_ARG;
  const int64_t TX = (int64_t)1 << tx_log2;
  const int64_t ctiles = (groups + TX - 1) / TX;
  // a small slab does not need all 1024 lanes: shrink the workgroup while 1 row per lane still covers it
  int block = kFusedBlock;
  while (block > 64 && block / 2 >= TX && (N + (block / 2) / TX - 1) / ((block / 2) / TX) <= 1) block /= 2;
  const int64_t TY = block / TX;
  const int64_t rows = (N + TY - 1) / TY;
  const int64_t blocks = ctiles > 1 ? (batch + kXcds - 1) / kXcds * kXcds * ctiles : batch;
  if (blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  const dim3 grid((uint32_t)blocks), blk(block);
  const bool nt = ctiles == 1 || TX >= 32;
#define KVQ_FUSED(R_)                                                                                               \
  do {                                                                                                              \
    if (nt)                                                                                                         \
      hipLaunchKernelGGL((fused_slab_kernel<R_, true>), grid, blk, 0, stream, x, scales, codes, batch, N, D, tx_log2, \
                         (uint32_t)ctiles);                                                                         \
    else                                                                                                            \
      hipLaunchKernelGGL((fused_slab_kernel<R_, false>), grid, blk, 0, stream, x, scales, codes, batch, N, D,       \
                         tx_log2, (uint32_t)ctiles);                                                                \
  } while (0)
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
