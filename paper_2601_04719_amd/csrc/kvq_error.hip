// Error statistics of the round trip
// (paper: Introduction, "Reconstruction error" and "Attention score error";
//  Evaluation, "Reconstruction Error" and "Attention Score Error").
//
//  - reconstruction error: sum of squares of the fp32 difference x - x_hat,
//    squared and summed in fp64, and the largest |x - x_hat|.
//  - attention-score error: mean over (query, token) of |q.k - q.k_hat|,
//    computed as |sum_d q_d (k_d - k_hat_d)| in fp64.
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
  int64_t blocks = (int64_t)dev.cus * options().blocks_per_cu;
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
  const Tiling t = make_tiling(batch, N, D, V, U, (int64_t)dev.cus * options().blocks_per_cu);
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
// A workgroup owns a tile of kTok tokens x kQry queries and walks the channel
// dimension in slices of kDc.  Each slice of e = k - k_hat and of the queries is
// staged in LDS as fp64; each lane keeps a 4 x 4 block of fp64 dot products.
constexpr int kTok = 64, kQry = 64, kDc = 32, kPad = 2;

template <bool FROM_CODES>
__global__ __launch_bounds__(kBlock) void attn_score_kernel(const float* __restrict__ queries, int64_t Q,
                                                            const float* __restrict__ k,
                                                            const float* __restrict__ k_hat,
                                                            const int8_t* __restrict__ codes,
                                                            const float* __restrict__ scales, int64_t N,
                                                            int64_t D, uint32_t qtiles, uint32_t tiles,
                                                            double* __restrict__ sums) {
  __shared__ double e_s[kDc][kTok + kPad];
  __shared__ double q_s[kDc][kQry + kPad];
  const int tid = threadIdx.x;
  const int tq = tid & 15;   // query block: queries 4*tq .. 4*tq+3
  const int tt = tid >> 4;   // token block: tokens 4*tt .. 4*tt+3
  // staging role: row `lr` of the tile (a token, or a query), channels lc .. lc+7 of the slice
  const int lr = tid >> 2;
  const int lc = (tid & 3) * 8;
  double total = 0.0;

  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int64_t q0 = (int64_t)(tile % qtiles) * kQry;
    const int64_t t0 = (int64_t)(tile / qtiles) * kTok;
    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < 4; b++) acc[a][b] = 0.0;

    for (int64_t d0 = 0; d0 < D; d0 += kDc) {
      const int64_t tok = t0 + lr, qry = q0 + lr;
#pragma unroll
      for (int i = 0; i < 8; i++) {
        const int64_t d = d0 + lc + i;
        double e = 0.0, qv = 0.0;
        if (d < D) {
          if (tok < N) {
            const float kv = k[tok * D + d];
            float kh;
            if constexpr (FROM_CODES) kh = (float)codes[tok * D + d] * scales[d];
            else kh = k_hat[tok * D + d];
            e = (double)kv - (double)kh;
          }
          if (qry < Q) qv = (double)queries[qry * D + d];
        }
        e_s[lc + i][lr] = e;
        q_s[lc + i][lr] = qv;
      }
      __syncthreads();
#pragma unroll 8
      for (int dd = 0; dd < kDc; dd++) {
        double ev[4], qv[4];
#pragma unroll
        for (int a = 0; a < 4; a++) ev[a] = e_s[dd][4 * tt + a];
#pragma unroll
        for (int b = 0; b < 4; b++) qv[b] = q_s[dd][4 * tq + b];
#pragma unroll
        for (int a = 0; a < 4; a++)
#pragma unroll
          for (int b = 0; b < 4; b++) acc[a][b] = fma(qv[b], ev[a], acc[a][b]);
      }
      __syncthreads();
    }
    // rows/queries outside the matrix were staged as zeros and contribute |0|
#pragma unroll
    for (int a = 0; a < 4; a++)
#pragma unroll
      for (int b = 0; b < 4; b++) total += fabs(acc[a][b]);
  }
  float unused = 0.0f;
  block_reduce(total, unused);
  if (tid == 0) sums[blockIdx.x] = total;
}

kvq_status launch_attn_score_error(const float* queries, int64_t Q, const float* k, const float* k_hat,
                                   const int8_t* codes, const float* scales, int64_t N, int64_t D,
                                   double* mean_abs_out, hipStream_t stream) {
  Workspace ws;
  if (kvq_status s = get_workspace(stream, &ws)) return s;
  const int64_t qtiles = (Q + kQry - 1) / kQry;
  const int64_t ttiles = (N + kTok - 1) / kTok;
  if (qtiles > INT32_MAX / 2 || ttiles > INT32_MAX / qtiles) return KVQ_ERR_OVERFLOW;
  const int64_t tiles = qtiles * ttiles;
  const int64_t blocks = tiles < kMaxPartials ? tiles : kMaxPartials;
  const dim3 grid((uint32_t)blocks), block(kBlock);
  if (k_hat)
    hipLaunchKernelGGL((attn_score_kernel<false>), grid, block, 0, stream, queries, Q, k, k_hat, codes, scales,
                       N, D, (uint32_t)qtiles, (uint32_t)tiles, ws.sums);
  else
    hipLaunchKernelGGL((attn_score_kernel<true>), grid, block, 0, stream, queries, Q, k, k_hat, codes, scales, N,
                       D, (uint32_t)qtiles, (uint32_t)tiles, ws.sums);
  KVQ_HIP(hipGetLastError());
  hipLaunchKernelGGL(fold_partials, dim3(1), dim3(kBlock), 0, stream, ws.sums, (const float*)nullptr,
                     (int)blocks, (double)Q * (double)N, mean_abs_out, (float*)nullptr);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
