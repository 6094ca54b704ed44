// Attention scores straight from the quantized cache:
//   scores[b,j,t] = sum_d q[b,j,d] * k_hat[b,t,d],   k_hat = (float)code * scale
// (paper: Background, Eq. (attention) -- the raw dot products q.k -- with the reconstruction of
//  Eq. (dequant_op); the integration direction named under "Future Work").
//
// This is what reads an int8 KV cache at decode time: a few queries per head against all cached
// keys.  The keys are never materialised in fp32: the scales are folded into the queries once per
// workgroup (qs = q * s, one fp32 rounding), and every code is used as read, so HBM traffic is
// 1 byte per cached element instead of 4.  A lane owns 16 adjacent channels (one 16-byte code load
// per row, contiguous across the lanes of a wavefront), keeps qs for them in registers, forms Q
// partial dot products per row in fp32 FMAs and the lanes of a row combine them with cross-lane
// shuffles.  Up to 8 queries per pass; more queries re-read the codes.
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

constexpr int kScoresMaxQ = 8;

// LLOG = log2(lanes per row).  D <= 16 << LLOG: one column chunk, the workgroup walks its rows in
// passes of TY * U rows with the folded queries resident in registers.  LLOG == 6 also serves
// D > 1024: then every pass over the rows is repeated per 1024-channel chunk (partial sums carried in
// registers), which re-reads the queries and scales per chunk -- the wide-D case is not the one a
// decode step meets.
template <int Q, int U, int LLOG>
__global__ __launch_bounds__(kBlock) void scores_kernel(const float* __restrict__ queries,
                                                        const int8_t* __restrict__ codes,
                                                        const float* __restrict__ scales,
                                                        float* __restrict__ out, int64_t N, int64_t D,
                                                        int64_t q_total, int64_t q_first, int q_count,
                                                        uint32_t rchunks, int64_t rows_per_chunk) {
  constexpr int L = 1 << LLOG;          // lanes per row
  constexpr int TY = kBlock >> LLOG;    // rows per workgroup pass
  const int tid = threadIdx.x;
  const int tx = tid & (L - 1);
  const int ty = tid >> LLOG;
  const int64_t slab = blockIdx.x / rchunks;
  const int64_t row0 = (int64_t)(blockIdx.x % rchunks) * rows_per_chunk;
  int64_t row1 = row0 + rows_per_chunk;
  if (row1 > N) row1 = N;
  const int8_t* cs = codes + slab * N * D;
  const float* ss = scales + slab * D;
  const float* qs_base = queries + (slab * q_total + q_first) * D;
  float* os = out + (slab * q_total + q_first) * N;
  const bool single = D <= (int64_t)16 * L;

  // the folded queries qs = q * s of this lane's 16 channels of column chunk c0
  auto fold = [&](int64_t col, bool active, float (&qs)[Q][16]) {
#pragma unroll
    for (int j = 0; j < Q; j++)
#pragma unroll
      for (int i = 0; i < 16; i++) qs[j][i] = 0.0f;
    if (active) {
      float s[16];
#pragma unroll
      for (int w = 0; w < 4; w++) {
        const f32x4 sv = *reinterpret_cast<const f32x4*>(ss + col + 4 * w);
        s[4 * w] = sv.x; s[4 * w + 1] = sv.y; s[4 * w + 2] = sv.z; s[4 * w + 3] = sv.w;
      }
#pragma unroll
      for (int j = 0; j < Q; j++) {
        if (j < q_count) {
#pragma unroll
          for (int w = 0; w < 4; w++) {
            const f32x4 qv = *reinterpret_cast<const f32x4*>(qs_base + (int64_t)j * D + col + 4 * w);
            qs[j][4 * w] = qv.x * s[4 * w];
            qs[j][4 * w + 1] = qv.y * s[4 * w + 1];
            qs[j][4 * w + 2] = qv.z * s[4 * w + 2];
            qs[j][4 * w + 3] = qv.w * s[4 * w + 3];
          }
        }
      }
    }
  };
  // U rows starting at r (TY apart): 16 codes per row and lane
  auto load_rows = [&](int64_t r, int64_t col, bool active, u32x4 (&cw)[U]) {
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int64_t rr = r + (int64_t)u * TY;
      cw[u] = u32x4{0u, 0u, 0u, 0u};
      if (active && rr < row1) cw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(cs + rr * D + col));
    }
  };
  // ... -> Q partial dot products per row
  auto dot_rows = [&](const u32x4 (&cw)[U], const float (&qs)[Q][16], float (&acc)[U][Q]) {
#pragma unroll
    for (int u = 0; u < U; u++)
#pragma unroll
      for (int w = 0; w < 4; w++) {
        const uint32_t word = cw[u][w];
#pragma unroll
        for (int b = 0; b < 4; b++) {
          const float c = (float)((int)(word << (24 - 8 * b)) >> 24);
#pragma unroll
          for (int j = 0; j < Q; j++) acc[u][j] = fmaf(qs[j][4 * w + b], c, acc[u][j]);
        }
      }
  };
  // combine the L lanes of each row; lane tx == 0 writes
  auto finish = [&](int64_t r, float (&acc)[U][Q]) {
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int64_t rr = r + (int64_t)u * TY;
#pragma unroll
      for (int j = 0; j < Q; j++) {
        float v = acc[u][j];
#pragma unroll
        for (int m = L >> 1; m > 0; m >>= 1) v += __shfl_xor(v, m, 64);
        if (tx == 0 && rr < row1 && j < q_count) os[(int64_t)j * N + rr] = v;
      }
    }
  };

  if (single) {
    const int64_t col = (int64_t)16 * tx;
    const bool active = col < D;
    float qs[Q][16];
    fold(col, active, qs);
    for (int64_t r = row0 + ty; r < row1; r += (int64_t)TY * U) {
      u32x4 cw[U];
      load_rows(r, col, active, cw);
      float acc[U][Q];
#pragma unroll
      for (int u = 0; u < U; u++)
#pragma unroll
        for (int j = 0; j < Q; j++) acc[u][j] = 0.0f;
      dot_rows(cw, qs, acc);
      finish(r, acc);
    }
  } else {
    for (int64_t r = row0 + ty; r < row1; r += (int64_t)TY * U) {
      float acc[U][Q];
#pragma unroll
      for (int u = 0; u < U; u++)
#pragma unroll
        for (int j = 0; j < Q; j++) acc[u][j] = 0.0f;
      for (int64_t c0 = 0; c0 < D; c0 += (int64_t)16 * L) {
        const int64_t col = c0 + (int64_t)16 * tx;
        const bool active = col < D;
        float qs[Q][16];
        fold(col, active, qs);
        u32x4 cw[U];
        load_rows(r, col, active, cw);
        dot_rows(cw, qs, acc);
      }
      finish(r, acc);
    }
  }
}

// Generic path (any D, any alignment): one lane per (row, query), scalar loads, same arithmetic
// order per lane as a single-lane row of the fast path.
__global__ __launch_bounds__(kBlock) void scores_generic_kernel(const float* __restrict__ queries,
                                                                const int8_t* __restrict__ codes,
                                                                const float* __restrict__ scales,
                                                                float* __restrict__ out, int64_t N, int64_t D,
                                                                int64_t Q, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= total) return;
  const int64_t t = i % N;
  const int64_t j = (i / N) % Q;
  const int64_t slab = i / (N * Q);
  const float* q = queries + (slab * Q + j) * D;
  const int8_t* c = codes + (slab * N + t) * D;
  const float* s = scales + slab * D;
  float acc = 0.0f;
  for (int64_t d = 0; d < D; d++) acc = fmaf(q[d] * s[d], (float)c[d], acc);
  out[i] = acc;
}

template <int Q, int LLOG>
static void launch_scores_ql(const float* queries, const int8_t* codes, const float* scales, float* out, int64_t N,
                             int64_t D, int64_t q_total, int64_t q_first, int q_count, int64_t batch, int cus,
                             hipStream_t stream) {
  constexpr int U = Q <= 2 ? 8 : 4;
  const int64_t pass_rows = (int64_t)(kBlock >> LLOG) * U;
  // passes per workgroup, from a sweep: short-lived workgroups stream best when a pass is cheap
  // (Q = 1), more passes amortise folding the scales into the queries when it is not; fewer when that
  // would leave under about 8 workgroups per compute unit
  int64_t passes = Q == 1 ? 2 : Q == 2 ? 8 : 16;
  while (passes > 1 && batch * ((N + pass_rows * passes - 1) / (pass_rows * passes)) < (int64_t)cus * 8) passes /= 2;
  const int64_t rows_per_chunk = pass_rows * passes;
  const int64_t rchunks = (N + rows_per_chunk - 1) / rows_per_chunk;
  hipLaunchKernelGGL((scores_kernel<Q, U, LLOG>), dim3((uint32_t)(batch * rchunks)), dim3(kBlock), 0, stream,
                     queries, codes, scales, out, N, D, q_total, q_first, q_count, (uint32_t)rchunks, rows_per_chunk);
}

template <int Q>
static void launch_scores_q(const float* queries, const int8_t* codes, const float* scales, float* out, int64_t N,
                            int64_t D, int64_t q_total, int64_t q_first, int q_count, int l_log2, int64_t batch,
                            int cus, hipStream_t stream) {
#define KVQ_SC(L_) \
  launch_scores_ql<Q, L_>(queries, codes, scales, out, N, D, q_total, q_first, q_count, batch, cus, stream)
  switch (l_log2) {
    case 0: KVQ_SC(0); break;
    case 1: KVQ_SC(1); break;
    case 2: KVQ_SC(2); break;
    case 3: KVQ_SC(3); break;
    case 4: KVQ_SC(4); break;
    case 5: KVQ_SC(5); break;
    default: KVQ_SC(6); break;
  }
#undef KVQ_SC
}

kvq_status launch_scores_from_codes(const float* queries, int64_t Q, const int8_t* codes, const float* scales,
                                    int64_t batch, int64_t N, int64_t D, float* out, hipStream_t stream) {
  // several queries per head: the int8 matrix-core kernel (no per-code vector ALU work)
  if (scores_mfma_applicable(queries, Q, codes, scales, D))
    return launch_scores_mfma(queries, Q, codes, scales, batch, N, D, out, stream);
  const bool fast = D % 16 == 0 && aligned(queries, 16) && aligned(codes, 16) && aligned(scales, 16);
  if (!fast) {
    const int64_t total = batch * Q * N;
    const int64_t blocks = (total + kBlock - 1) / kBlock;
    if (blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
    hipLaunchKernelGGL(scores_generic_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0, stream, queries, codes,
                       scales, out, N, D, Q, total);
    KVQ_HIP(hipGetLastError());
    return KVQ_OK;
  }
  int l_log2 = 0;
  while ((1 << l_log2) < 64 && ((int64_t)16 << l_log2) < D) l_log2++;
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  const int64_t TY = kBlock >> l_log2;
  const int64_t rchunks = (N + TY * 4 - 1) / (TY * 4);
  if (batch * rchunks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  for (int64_t q0 = 0; q0 < Q; q0 += kScoresMaxQ) {
    const int qc = (int)(Q - q0 < kScoresMaxQ ? Q - q0 : kScoresMaxQ);
    if (qc == 1) launch_scores_q<1>(queries, codes, scales, out, N, D, Q, q0, qc, l_log2, batch, dev.cus, stream);
    else if (qc == 2) launch_scores_q<2>(queries, codes, scales, out, N, D, Q, q0, qc, l_log2, batch, dev.cus, stream);
    else if (qc <= 4) launch_scores_q<4>(queries, codes, scales, out, N, D, Q, q0, qc, l_log2, batch, dev.cus, stream);
    else launch_scores_q<8>(queries, codes, scales, out, N, D, Q, q0, qc, l_log2, batch, dev.cus, stream);
    KVQ_HIP(hipGetLastError());
  }
  return KVQ_OK;
}

}  // namespace kvq
