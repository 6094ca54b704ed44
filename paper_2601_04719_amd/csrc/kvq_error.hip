// Error statistics of the round trip
// (paper: Introduction, "Reconstruction error" and "Attention score error";
//  Evaluation, "Reconstruction Error" and "Attention Score Error").
//
//  - reconstruction error: sum of squares of the fp32 difference x - x_hat,
//    squared and summed in fp64, and the largest |x - x_hat|.
//  - attention-score error: mean over (query, token) of |q.k - q.k_hat|,
//    computed as |sum_d q_d (k_d - k_hat_d)| in fp64 on the fp64 matrix cores.
//
// Reductions are two-level and order-fixed: every workgroup writes one partial
// (sum, max) into a per-stream workspace, and a single-workgroup kernel folds
// the partials in index order, so a given shape always gives the same bits.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

// ---------------------------------------------------------------- reductions
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_down(v, off, 64));
  return v;
}

// Workgroup-wide (sum, max); the result is valid in thread 0.
__device__ __forceinline__ void block_reduce(double& sum, float& mx) {
  __shared__ double s_sum[kBlock / 64];
  __shared__ float s_max[kBlock / 64];
  sum = wave_sum(sum);
  mx = wave_max(mx);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) {
    s_sum[wave] = sum;
    s_max[wave] = mx;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kBlock / 64; w++) {
      sum += s_sum[w];
      mx = fmaxf(mx, s_max[w]);
    }
  }
}

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

// ------------------------------------------------------ attention-score error
// The score difference  q_j . k_t - q_j . k_hat_t = sum_d q_j[d] (k_t[d] - k_hat_t[d])  is a dense
// [tokens x D] . [D x queries] contraction in fp64, so it runs on the fp64 matrix cores
// (v_mfma_f64_16x16x4_f64).
//
// A workgroup (4 wavefronts) owns 64 tokens x 16*NQ queries and walks D in chunks of kDc channels.
// Per chunk it stages e = (double)k - (double)k_hat [64 x kDc] and the queries [16*NQ x kDc] in LDS
// as fp64 (converted once, with 256-byte coalesced global reads), double-buffered: the global loads
// of chunk c+1 are in flight while chunk c is contracted, one barrier per chunk.  Wavefront w owns
// tokens 16w..16w+15 and NQ accumulator tiles.  For each block of 16 channels, lane (r = lane % 16,
// g = lane / 16) reads channels 4g..4g+3 of token r and of query r of every query tile from LDS and
// feeds four MFMA steps; step c contracts channels {4g + c : g = 0..3}.  Only sum |C| over the
// accumulator tiles is needed, so where C elements sit in registers does not matter.  Tokens,
// queries and channels outside the matrices are staged as zeros and add |0|.
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));

constexpr int kTok = 64;  // tokens per workgroup

struct Quad {
  float v[4];
};

// four consecutive floats p[idx..idx+3] of a row (vector load when VEC), zero where idx + i >= limit or !ok
template <bool VEC>
__device__ __forceinline__ Quad load_quad(const float* __restrict__ row, int64_t idx, int64_t limit, bool ok) {
  Quad q;
  if constexpr (VEC) {
    f32x4 t = {0.f, 0.f, 0.f, 0.f};
    if (ok && idx < limit) t = *reinterpret_cast<const f32x4*>(row + idx);
    q.v[0] = t.x; q.v[1] = t.y; q.v[2] = t.z; q.v[3] = t.w;
  } else {
#pragma unroll
    for (int i = 0; i < 4; i++) q.v[i] = (ok && idx + i < limit) ? row[idx + i] : 0.0f;
  }
  return q;
}

// same for the reconstructed key: either read, or recomputed as (float)code * scale
template <bool VEC, bool FROM_CODES>
__device__ __forceinline__ Quad load_khat(const float* __restrict__ k_hat, const int8_t* __restrict__ codes,
                                          const float* __restrict__ scales, int64_t row_off, int64_t d, int64_t D,
                                          bool ok) {
  if constexpr (!FROM_CODES) {
    return load_quad<VEC>(k_hat + row_off, d, D, ok);
  } else {
    Quad q;
    if constexpr (VEC) {
      uint32_t w = 0;
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
      if (ok && d < D) {
        w = *reinterpret_cast<const uint32_t*>(codes + row_off + d);
        s = *reinterpret_cast<const f32x4*>(scales + d);
      }
#pragma unroll
      for (int i = 0; i < 4; i++) q.v[i] = (float)((int)(w << (24 - 8 * i)) >> 24) * s[i];
    } else {
#pragma unroll
      for (int i = 0; i < 4; i++)
        q.v[i] = (ok && d + i < D) ? (float)codes[row_off + d + i] * scales[d + i] : 0.0f;
    }
    return q;
  }
}

// kDc = channels per staged chunk: 32 lets two workgroups share a compute unit's LDS (they overlap each
// other's staging); 64 halves the barriers and is the better choice when there is at most one
// workgroup per compute unit anyway.
template <int NQ, int kDc, bool VEC, bool FROM_CODES>
__global__ __launch_bounds__(kBlock) void attn_score_kernel(const float* __restrict__ queries, int64_t Q,
                                                            const float* __restrict__ k,
                                                            const float* __restrict__ k_hat,
                                                            const int8_t* __restrict__ codes,
                                                            const float* __restrict__ scales, int64_t N,
                                                            int64_t D, uint32_t qchunks, uint32_t tiles,
                                                            double* __restrict__ sums) {
  constexpr int kPitch = kDc + 2;                // LDS row pitch in doubles: 16-byte skew between rows
  constexpr int QR = 16 * NQ;                    // query rows staged per chunk
  constexpr int F4 = kDc / 4;                    // 16-byte pieces per staged row
  constexpr int ROWS_PER_PASS = kBlock / F4;     // rows one fill pass of the workgroup covers
  constexpr int KP = kTok / ROWS_PER_PASS;       // fill passes for the token rows
  constexpr int QP = (QR + ROWS_PER_PASS - 1) / ROWS_PER_PASS;
  __shared__ double e_s[2][kTok][kPitch];
  __shared__ double q_s[2][QR][kPitch];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15;   // row of the 16-row operand tile: a token (A operand) or a query (B operand)
  const int g = lane >> 4;   // which 4 of a block's 16 channels this lane supplies
  const int frow = tid / F4; // fill role: row within a pass, and which 16-byte piece of the chunk
  const int fcol = (tid % F4) * 4;
  double total = 0.0;

  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int64_t q0 = (int64_t)(tile % qchunks) * QR;
    const int64_t t0 = (int64_t)(tile / qchunks) * kTok;
    f64x4 acc[NQ];
#pragma unroll
    for (int n = 0; n < NQ; n++) acc[n] = f64x4{0.0, 0.0, 0.0, 0.0};

    Quad kv[KP], hv[KP], qv[QP];
    auto fetch = [&](int64_t d0) {
      const int64_t d = d0 + fcol;
#pragma unroll
      for (int p = 0; p < KP; p++) {
        const int64_t tok = t0 + frow + p * ROWS_PER_PASS;
        kv[p] = load_quad<VEC>(k + tok * D, d, D, tok < N);
        hv[p] = load_khat<VEC, FROM_CODES>(k_hat, codes, scales, tok * D, d, D, tok < N);
      }
#pragma unroll
      for (int p = 0; p < QP; p++) {
        const int row = frow + p * ROWS_PER_PASS;
        const int64_t qi = q0 + row;
        qv[p] = load_quad<VEC>(queries + qi * D, d, D, row < QR && qi < Q);
      }
    };
    auto stage = [&](int buf) {
#pragma unroll
      for (int p = 0; p < KP; p++) {
        double* dst = &e_s[buf][frow + p * ROWS_PER_PASS][fcol];
        f64x2 lo = {(double)kv[p].v[0] - (double)hv[p].v[0], (double)kv[p].v[1] - (double)hv[p].v[1]};
        f64x2 hi = {(double)kv[p].v[2] - (double)hv[p].v[2], (double)kv[p].v[3] - (double)hv[p].v[3]};
        *reinterpret_cast<f64x2*>(dst) = lo;
        *reinterpret_cast<f64x2*>(dst + 2) = hi;
      }
#pragma unroll
      for (int p = 0; p < QP; p++) {
        const int row = frow + p * ROWS_PER_PASS;
        if (row < QR) {
          double* dst = &q_s[buf][row][fcol];
          f64x2 lo = {(double)qv[p].v[0], (double)qv[p].v[1]};
          f64x2 hi = {(double)qv[p].v[2], (double)qv[p].v[3]};
          *reinterpret_cast<f64x2*>(dst) = lo;
          *reinterpret_cast<f64x2*>(dst + 2) = hi;
        }
      }
    };

    __syncthreads();  // the previous tile's last chunk has been consumed by every wavefront
    fetch(0);
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int64_t d0 = 0; d0 < D; d0 += kDc, buf ^= 1) {
      const bool more = d0 + kDc < D;
      if (more) fetch(d0 + kDc);
      // operands of block b+1 are read from LDS before the MFMAs of block b are issued
      double e[4], qd[NQ][4];
      auto read_block = [&](int b, double (&e_)[4], double (&q_)[NQ][4]) {
        const double* ep = &e_s[buf][16 * wave + r][16 * b + 4 * g];
        const f64x2 e01 = *reinterpret_cast<const f64x2*>(ep);
        const f64x2 e23 = *reinterpret_cast<const f64x2*>(ep + 2);
        e_[0] = e01.x; e_[1] = e01.y; e_[2] = e23.x; e_[3] = e23.y;
#pragma unroll
        for (int n = 0; n < NQ; n++) {
          const double* qp = &q_s[buf][16 * n + r][16 * b + 4 * g];
          const f64x2 q01 = *reinterpret_cast<const f64x2*>(qp);
          const f64x2 q23 = *reinterpret_cast<const f64x2*>(qp + 2);
          q_[n][0] = q01.x; q_[n][1] = q01.y; q_[n][2] = q23.x; q_[n][3] = q23.y;
        }
      };
      read_block(0, e, qd);
#pragma unroll
      for (int b = 0; b < kDc / 16; b++) {
        double e_n[4], qd_n[NQ][4];
        if (b + 1 < kDc / 16) read_block(b + 1, e_n, qd_n);
#pragma unroll
        for (int c = 0; c < 4; c++)
#pragma unroll
          for (int n = 0; n < NQ; n++)
            acc[n] = __builtin_amdgcn_mfma_f64_16x16x4f64(e[c], qd[n][c], acc[n], 0, 0, 0);
        if (b + 1 < kDc / 16) {
#pragma unroll
          for (int c = 0; c < 4; c++) {
            e[c] = e_n[c];
#pragma unroll
            for (int n = 0; n < NQ; n++) qd[n][c] = qd_n[n][c];
          }
        }
      }
      if (more) stage(buf ^ 1);
      __syncthreads();
    }
#pragma unroll
    for (int n = 0; n < NQ; n++)
#pragma unroll
      for (int i = 0; i < 4; i++) total += fabs(acc[n][i]);
  }
  float unused = 0.0f;
  block_reduce(total, unused);
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

kvq_status launch_attn_score_error(const float* queries, int64_t Q, const float* k, const float* k_hat,
                                   const int8_t* codes, const float* scales, int64_t N, int64_t D,
                                   double* mean_abs_out, hipStream_t stream) {
  Workspace ws;
  if (kvq_status s = get_workspace(stream, &ws)) return s;
  const int NQ = Q > 32 ? 4 : Q > 16 ? 2 : 1;          // query tiles of 16 per workgroup
  const int64_t qchunks = (Q + 16 * NQ - 1) / (16 * NQ);
  const int64_t ttiles = (N + kTok - 1) / kTok;
  if (qchunks > INT32_MAX / 2 || ttiles > INT32_MAX / qchunks) return KVQ_ERR_OVERFLOW;
  const int64_t tiles = qchunks * ttiles;
  const int64_t blocks = tiles < kMaxPartials ? tiles : kMaxPartials;
  const bool from_codes = k_hat == nullptr;
  bool vec = D % 4 == 0 && aligned(queries, 16) && aligned(k, 16);
  vec = vec && (from_codes ? (aligned(codes, 4) && aligned(scales, 16)) : aligned(k_hat, 16));
  const dim3 grid((uint32_t)blocks), block(kBlock);
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  const bool wide = tiles <= (int64_t)dev.cus;   // at most one workgroup per compute unit: long chunks
#define KVQ_LAUNCH_AS(NQ_, DC_, VEC_, FC_)                                                                      \
  hipLaunchKernelGGL((attn_score_kernel<NQ_, DC_, VEC_, FC_>), grid, block, 0, stream, queries, Q, k, k_hat,    \
                     codes, scales, N, D, (uint32_t)qchunks, (uint32_t)tiles, ws.sums)
#define KVQ_PICK_AS(NQ_)                                                 \
  do {                                                                   \
    if (vec && from_codes && wide) KVQ_LAUNCH_AS(NQ_, 64, true, true);   \
    else if (vec && from_codes) KVQ_LAUNCH_AS(NQ_, 32, true, true);      \
    else if (vec && wide) KVQ_LAUNCH_AS(NQ_, 64, true, false);           \
    else if (vec) KVQ_LAUNCH_AS(NQ_, 32, true, false);                   \
    else if (from_codes) KVQ_LAUNCH_AS(NQ_, 32, false, true);            \
    else KVQ_LAUNCH_AS(NQ_, 32, false, false);                           \
  } while (0)
  if (NQ == 4) KVQ_PICK_AS(4);
  else if (NQ == 2) KVQ_PICK_AS(2);
  else KVQ_PICK_AS(1);
#undef KVQ_PICK_AS
#undef KVQ_LAUNCH_AS
  KVQ_HIP(hipGetLastError());
  hipLaunchKernelGGL(fold_partials, dim3(1), dim3(kBlock), 0, stream, ws.sums, (const float*)nullptr,
                     (int)blocks, (double)Q * (double)N, mean_abs_out, (float*)nullptr);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
