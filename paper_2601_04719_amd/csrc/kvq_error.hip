// Reconstruction error of the round trip
// (paper: Introduction, "Reconstruction error"; Evaluation, "Reconstruction Error"):
// sum of squares of the fp32 difference x - x_hat, squared and summed in fp64, and
// the largest |x - x_hat|.
//
// Reductions are two-level and order-fixed: every workgroup writes one partial
// (sum, max) into a per-stream workspace, and a single-workgroup kernel folds
// the partials in index order, so a given shape always gives the same bits.
#include <type_traits>

#include "kvq_internal.h"
#include "kvq_reduce.h"

namespace kvq {

// Folds n partials in index order.  sum_out = sum * sum_scale; max_out may be NULL.
__global__ __launch_bounds__(kBlock) void fold_partials(const double* __restrict__ sums,
                                                        const float* __restrict__ maxes, int n,
                                                        double divisor, double* __restrict__ sum_out,
                                                        float* __restrict__ max_out) {
  double s = 0.0;
  float m = 0.0f;
  for (int i = threadIdx.x; i < n; i += kBlock) {
    s += sums[i];
    if (maxes) m = fmaxf(m, maxes[i]);
  }
  block_reduce(s, m);
  if (threadIdx.x == 0) {
    *sum_out = s / divisor;
    if (max_out) *max_out = m;
  }
}

__device__ __forceinline__ void err_step(float x, float xh, double& acc, float& mx) {
  const float e = x - xh;            // fp32 difference, as the matrices are fp32
  const double ed = (double)e;
  acc = fma(ed, ed, acc);            // the square of an fp32 value is exact in fp64: same bits as mul, add
  mx = fmaxf(mx, fabsf(e));
}

// ------------------------------------------- reconstruction error, x vs x_hat
// Flat stream over `count` elements; VEC = 4 needs both pointers 16-byte aligned.
// Every workgroup owns one contiguous chunk of `chunk` vectors (a multiple of
// kBlock * U) and walks it front to back with U consecutive 4 KiB tiles of each
// matrix in flight.
template <int VEC, int U>
__global__ __launch_bounds__(kBlock) void roundtrip_dense_kernel(const float* __restrict__ x,
                                                                 const float* __restrict__ xh, int64_t count,
                                                                 int64_t chunk, double* __restrict__ sums,
                                                                 float* __restrict__ maxes) {
  double acc[VEC];
  float mx = 0.0f;
#pragma unroll
  for (int i = 0; i < VEC; i++) acc[i] = 0.0;
  const int64_t nvec = count / VEC;
  int64_t i = (int64_t)blockIdx.x * chunk + threadIdx.x;
  int64_t end = (int64_t)(blockIdx.x + 1) * chunk;
  if (end > nvec) end = nvec;
  if constexpr (VEC == 4) {
    const f32x4* xv = reinterpret_cast<const f32x4*>(x);
    const f32x4* hv = reinterpret_cast<const f32x4*>(xh);
    for (; i + (int64_t)(U - 1) * kBlock < end; i += (int64_t)U * kBlock) {
      f32x4 a[U], b[U];
#pragma unroll
      for (int u = 0; u < U; u++) {
        a[u] = ld<true>(xv + i + u * kBlock);
        b[u] = ld<true>(hv + i + u * kBlock);
      }
#pragma unroll
      for (int u = 0; u < U; u++) {
        err_step(a[u].x, b[u].x, acc[0], mx);
        err_step(a[u].y, b[u].y, acc[1], mx);
        err_step(a[u].z, b[u].z, acc[2], mx);
        err_step(a[u].w, b[u].w, acc[3], mx);
      }
    }
    for (; i < end; i += kBlock) {
      const f32x4 a = xv[i], b = hv[i];
      err_step(a.x, b.x, acc[0], mx);
      err_step(a.y, b.y, acc[1], mx);
      err_step(a.z, b.z, acc[2], mx);
      err_step(a.w, b.w, acc[3], mx);
    }
    // the count % 4 trailing elements
    if (blockIdx.x == 0 && threadIdx.x < count - nvec * 4) {
      const int64_t j = nvec * 4 + threadIdx.x;
      err_step(x[j], xh[j], acc[0], mx);
    }
  } else {
    for (; i < end; i += kBlock) err_step(x[i], xh[i], acc[0], mx);
  }
  double sum = acc[0];
#pragma unroll
  for (int k = 1; k < VEC; k++) sum += acc[k];
  block_reduce(sum, mx);
  if (threadIdx.x == 0) {
    sums[blockIdx.x] = sum;
    maxes[blockIdx.x] = mx;
  }
}

// ------------------------------- reconstruction error, x vs codes and scales
// Same lane layout as the dequantize kernel; x_hat = (float)code * scale is
// formed in fp32 exactly as dequantize forms it, never stored.
template <int V, int U>
__global__ __launch_bounds__(kBlock) void roundtrip_codes_kernel(const float* __restrict__ x,
                                                                 const int8_t* __restrict__ codes,
                                                                 const float* __restrict__ scales, int64_t N,
                                                                 int64_t D, int tx_log2, uint32_t ctiles,
                                                                 uint32_t rchunks, int64_t rows_per_chunk,
                                                                 int64_t groups, uint32_t items,
                                                                 double* __restrict__ sums,
                                                                 float* __restrict__ maxes) {
  constexpr int A = V >= 4 ? 4 : 1;
  double acc[A];
  float mx = 0.0f;
#pragma unroll
  for (int i = 0; i < A; i++) acc[i] = 0.0;

  for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
    const Item it = decode_item(item, ctiles, rchunks, rows_per_chunk, N, tx_log2);
    if (it.group >= groups) continue;
    const int64_t col = it.group * V;
    float s[V];
    const float* sp = scales + it.slab * D + col;
#pragma unroll
    for (int i = 0; i < V; i++) s[i] = sp[i];
    const int64_t step = (int64_t)it.TY * D;
    int64_t row = it.row0 + it.ty;
    const float* px = x + (it.slab * N + row) * D + col;
    const int8_t* pc = codes + (it.slab * N + row) * D + col;
    if constexpr (V >= 4) {
      constexpr int W = V / 4;
      typedef typename std::conditional<V == 16, u32x4, typename std::conditional<V == 8, u32x2, uint32_t>::type>::type cvec;
      auto do_rows = [&](auto tag) {
        constexpr int R = decltype(tag)::value;
        f32x4 v[R][W];
        cvec c[R];
#pragma unroll
        for (int u = 0; u < R; u++) {
          c[u] = ld<true>(reinterpret_cast<const cvec*>(pc + u * step));
#pragma unroll
          for (int w = 0; w < W; w++) v[u][w] = ld<true>(reinterpret_cast<const f32x4*>(px + u * step) + w);
        }
#pragma unroll
        for (int u = 0; u < R; u++)
#pragma unroll
          for (int w = 0; w < W; w++) {
            uint32_t word;
            if constexpr (V == 4) word = c[u];
            else word = c[u][w];
#pragma unroll
            for (int b = 0; b < 4; b++) {
              const int q = (int)(word << (24 - 8 * b)) >> 24;
              const float xh = (float)q * s[4 * w + b];
              err_step(v[u][w][b], xh, acc[b], mx);
            }
          }
      };
      for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, px += U * step, pc += U * step)
        do_rows(std::integral_constant<int, U>{});
      for (; row < it.row1; row += it.TY, px += step, pc += step) do_rows(std::integral_constant<int, 1>{});
    } else {
      for (; row < it.row1; row += it.TY, px += step, pc += step) {
        const float xh = (float)(*pc) * s[0];
        err_step(*px, xh, acc[0], mx);
      }
    }
  }
  double sum = acc[0];
#pragma unroll
  for (int k = 1; k < A; k++) sum += acc[k];
  block_reduce(sum, mx);
  if (threadIdx.x == 0) {
    sums[blockIdx.x] = sum;
    maxes[blockIdx.x] = mx;
  }
}

// Wide rows (D >= 2048 channels): the lanes of a workgroup own J column groups each, 256 groups apart,
// so that the workgroup reads whole rows -- one fat contiguous stream of x and one of codes per
// workgroup, as in the scale reduction -- with the J * 4 scales of a lane in registers.
template <int J>
__global__ __launch_bounds__(kBlock) void roundtrip_codes_rows_kernel(const float* __restrict__ x,
                                                                      const int8_t* __restrict__ codes,
                                                                      const float* __restrict__ scales, int64_t N,
                                                                      int64_t D, uint32_t ctiles, uint32_t rchunks,
                                                                      int64_t rows_per_chunk, int64_t groups,
                                                                      uint32_t items, double* __restrict__ sums,
                                                                      float* __restrict__ maxes) {
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  float mx = 0.0f;
  for (uint32_t item = blockIdx.x; item < items; item += gridDim.x) {
    const uint32_t ct = item % ctiles, rest = item / ctiles;
    const uint32_t rc = rest % rchunks;
    const int64_t slab = rest / rchunks;
    const int64_t group0 = (int64_t)ct * kBlock * J + threadIdx.x;
    const int64_t row0 = (int64_t)rc * rows_per_chunk;
    int64_t row1 = row0 + rows_per_chunk;
    if (row1 > N) row1 = N;
    f32x4 s[J];
    bool act[J];
#pragma unroll
    for (int j = 0; j < J; j++) {
      act[j] = group0 + (int64_t)j * kBlock < groups;
      s[j] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (act[j]) s[j] = *reinterpret_cast<const f32x4*>(scales + slab * D + (group0 + (int64_t)j * kBlock) * 4);
    }
    const float* px = x + (slab * N + row0) * D + group0 * 4;
    const int8_t* pc = codes + (slab * N + row0) * D + group0 * 4;
    // U = 8 / J rows at a time: eight 16-byte and eight 4-byte loads in flight per lane
    constexpr int U = 8 / J;
    auto do_rows = [&](auto tag) {
      constexpr int R = decltype(tag)::value;
      f32x4 v[R][J];
      uint32_t w[R][J];
#pragma unroll
      for (int u = 0; u < R; u++)
#pragma unroll
        for (int j = 0; j < J; j++) {
          v[u][j] = f32x4{0.f, 0.f, 0.f, 0.f};
          w[u][j] = 0u;
          if (act[j]) {
            v[u][j] = ld<true>(reinterpret_cast<const f32x4*>(px + u * D) + (int64_t)j * kBlock);
            w[u][j] = ld<true>(reinterpret_cast<const uint32_t*>(pc + u * D) + (int64_t)j * kBlock);
          }
        }
#pragma unroll
      for (int u = 0; u < R; u++)
#pragma unroll
        for (int j = 0; j < J; j++)
#pragma unroll
          for (int b = 0; b < 4; b++) {
            const int q = (int)(w[u][j] << (24 - 8 * b)) >> 24;
            const float xh = (float)q * s[j][b];   // inactive groups: 0 * 0 against x = 0
            err_step(v[u][j][b], xh, acc[b], mx);
          }
    };
    int64_t row = row0;
    for (; row + U <= row1; row += U, px += U * D, pc += U * D) do_rows(std::integral_constant<int, U>{});
    for (; row < row1; row++, px += D, pc += D) do_rows(std::integral_constant<int, 1>{});
  }
  double sum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
  block_reduce(sum, mx);
  if (threadIdx.x == 0) {
    sums[blockIdx.x] = sum;
    maxes[blockIdx.x] = mx;
  }
}

kvq_status launch_roundtrip_error_dense(const float* x, const float* x_hat, int64_t count, double* sumsq_out,
                                        float* maxabs_out, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  Workspace ws;
  if (kvq_status s = get_workspace(stream, &ws)) return s;
  constexpr int U = 4;
  const bool vec = aligned(x, 16) && aligned(x_hat, 16);
  const int64_t work = vec ? count / 4 : count;           // vectors (or elements) to walk
  const int64_t tile = (int64_t)kBlock * U;
  // one long contiguous chunk per compute unit: as for the scale reduction, a read-only stream runs best as
  // one fat walk per unit (1 / 2 / 8 workgroups per unit: 7.24 / 7.15 / 7.06 TB/s on [131072 x 8192],
  // 6.94 / 6.76 / 6.60 on [16384 x 8192])
  const int per_cu = options().blocks_per_cu > 0 ? options().blocks_per_cu : 1;
  int64_t blocks = (int64_t)dev.cus * per_cu;
  if (blocks > kMaxPartials) blocks = kMaxPartials;
  int64_t chunk = (work + blocks - 1) / blocks;
  chunk = (chunk + tile - 1) / tile * tile;
  if (chunk < tile) chunk = tile;
  blocks = (work + chunk - 1) / chunk;
  if (blocks < 1) blocks = 1;
  if (vec)
    hipLaunchKernelGGL((roundtrip_dense_kernel<4, U>), dim3((uint32_t)blocks), dim3(kBlock), 0, stream, x, x_hat,
                       count, chunk, ws.sums, ws.maxes);
  else
    hipLaunchKernelGGL((roundtrip_dense_kernel<1, U>), dim3((uint32_t)blocks), dim3(kBlock), 0, stream, x, x_hat,
                       count, chunk, ws.sums, ws.maxes);
  KVQ_HIP(hipGetLastError());
  hipLaunchKernelGGL(fold_partials, dim3(1), dim3(kBlock), 0, stream, ws.sums, ws.maxes, (int)blocks, 1.0,
                     sumsq_out, maxabs_out);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

kvq_status launch_roundtrip_error_codes(const float* x, const int8_t* codes, const float* scales,
                                        int64_t batch, int64_t N, int64_t D, double* sumsq_out,
                                        float* maxabs_out, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  Workspace ws;
  if (kvq_status s = get_workspace(stream, &ws)) return s;
  constexpr int U = 4;
  // 4 channels per lane, as in the codec kernels: every wavefront access is one contiguous segment
  int V = pick_width(D, x, codes, 4);
  if (V > 1 && !aligned(scales, 16)) V = 1;
  if (V == 4 && D >= 2048) {
    // rows at least two workgroup-widths wide: row-spanning lanes, one or two workgroups per compute unit
    const int64_t groups = D / 4;
    int J = 1;
    while (J < 8 && (int64_t)kBlock * J * 2 <= groups) J *= 2;
    const int64_t ctiles = (groups + (int64_t)kBlock * J - 1) / ((int64_t)kBlock * J);
    const int per_cu = options().blocks_per_cu > 0 ? options().blocks_per_cu : 2;
    int64_t want = ((int64_t)dev.cus * per_cu + batch * ctiles - 1) / (batch * ctiles);
    if (want < 1) want = 1;
    if (want > N) want = N;
    const int64_t rows = (N + want - 1) / want;
    const int64_t rchunks = (N + rows - 1) / rows;
    const int64_t items = batch * rchunks * ctiles;
    if (items > INT32_MAX) return KVQ_ERR_OVERFLOW;
    const int64_t nblocks = items < kMaxPartials ? items : kMaxPartials;
    const dim3 grid((uint32_t)nblocks), block(kBlock);
#define KVQ_LAUNCH_RR(J_)                                                                                       \
  hipLaunchKernelGGL((roundtrip_codes_rows_kernel<J_>), grid, block, 0, stream, x, codes, scales, N, D,         \
                     (uint32_t)ctiles, (uint32_t)rchunks, rows, groups, (uint32_t)items, ws.sums, ws.maxes)
    if (J == 8) KVQ_LAUNCH_RR(8);
    else if (J == 4) KVQ_LAUNCH_RR(4);
    else KVQ_LAUNCH_RR(2);
#undef KVQ_LAUNCH_RR
    KVQ_HIP(hipGetLastError());
    hipLaunchKernelGGL(fold_partials, dim3(1), dim3(kBlock), 0, stream, ws.sums, ws.maxes, (int)nblocks, 1.0,
                       sumsq_out, maxabs_out);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
  }
  // two workgroups per compute unit (1 / 2 / 8: 6.61 / 6.82 / 6.67 TB/s on [131072 x 8192], 6.07 / 6.10 / 5.69
  // on [16384 x 8192], 6.06 / 6.64 / 6.47 on [256 x 4096 x 128])
  const int per_cu = options().blocks_per_cu > 0 ? options().blocks_per_cu : 2;
  const Tiling t = make_tiling(batch, N, D, V, U, (int64_t)dev.cus * per_cu);
  if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
  int64_t blocks = t.items < kMaxPartials ? t.items : kMaxPartials;
  const dim3 grid((uint32_t)blocks), block(kBlock);
#define KVQ_LAUNCH_RC(V_)                                                                                  \
  hipLaunchKernelGGL((roundtrip_codes_kernel<V_, U>), grid, block, 0, stream, x, codes, scales, N, D,      \
                     t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups, (uint32_t)t.items, ws.sums, \
                     ws.maxes)
  if (V == 4) KVQ_LAUNCH_RC(4);
  else KVQ_LAUNCH_RC(1);
#undef KVQ_LAUNCH_RC
  KVQ_HIP(hipGetLastError());
  hipLaunchKernelGGL(fold_partials, dim3(1), dim3(kBlock), 0, stream, ws.sums, ws.maxes, (int)blocks, 1.0,
                     sumsq_out, maxabs_out);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

kvq_status launch_fold_partials(const double* sums, const float* maxes, int n, double divisor, double* sum_out,
                                float* max_out, hipStream_t stream) {
  hipLaunchKernelGGL(fold_partials, dim3(1), dim3(kBlock), 0, stream, sums, maxes, n, divisor, sum_out, max_out);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
