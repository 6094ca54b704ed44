// Attention scores straight from a 4-bit cache (two codes per byte, scales = absmax / 7):
//   scores[b,j,t] = sum_d (q[b,j,d] * s[b,d]) * code[b,t,d],  code in [-7, 7]
// (paper: Background, Eq. (attention) with the reconstruction of Eq. (dequant_op); Limitations,
//  "Lower bit-widths"; Future Work, integration into attention).
//
// Same construction as the int8 matrix-core kernel: the folded queries become four int8 digits of a
// 28-bit fixed-point number, the integer dot products are exact, one rounding at the end.  What is
// new is how the packed codes become an MFMA operand without sign extension: a 32-bit word of eight
// nibbles is XORed with 0x88888888, which turns every two's-complement nibble q into q + 8 (1..15),
// and split into its even nibbles (w & 0x0F0F0F0F) and odd nibbles ((w >> 4) & 0x0F0F0F0F) -- two
// words of four small non-negative bytes each.  The constant offset is taken out exactly afterwards:
//   sum_d I[d] * q[d] = sum_d I[d] * (q[d] + 8) - 8 * sum_d I[d],
// all integers (the second sum is formed once per query).  The digits are stored in the channel
// order this split produces (even channels of a word, then its odd channels), so nothing is permuted
// at run time.  HBM traffic is half a byte per cached element; the vector ALUs spend four operations
// per eight codes.
//
// A lane loads 16 packed bytes (32 channels) per token and double step, feeding two MFMA steps.
// Needs D % 128 == 0, D <= 1024 and 16-byte aligned packed rows; other shapes take a scalar kernel.
#include "kvq_internal.h"

namespace kvq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// position (0..15) of channel c (0..15) of a lane's half-load inside the MFMA operand
__device__ __forceinline__ int nibble_pos(int c) {
  const int w = c >> 3, k = c & 7;  // word, nibble within the word
  return 8 * w + 4 * (k & 1) + (k >> 1);
}

template <int G>
__global__ __launch_bounds__(kBlock) void scores_int4_mfma_kernel(const float* __restrict__ queries,
                                                                  const uint8_t* __restrict__ packed,
                                                                  const float* __restrict__ scales,
                                                                  float* __restrict__ out, int64_t N, int64_t D,
                                                                  int64_t q_total, int64_t q_first, int q_count,
                                                                  uint32_t chunks, int64_t tokens_per_chunk) {
  constexpr int TU = 4;
  extern __shared__ __align__(16) unsigned char lds[];
  const int dsteps = (int)(D >> 7);  // double steps of 128 channels
  // [dsteps][2][G][64 lanes][16 bytes] digits, then per query: 2^(E-27) and sum_d I[d] (both fp64, exact)
  unsigned char* dig = lds;
  double* qscale = reinterpret_cast<double*>(lds + (size_t)dsteps * 2 * G * 1024);
  double* qsum = qscale + 4 * G;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int64_t slab = blockIdx.x / chunks;
  const int64_t t_begin = (int64_t)(blockIdx.x % chunks) * tokens_per_chunk;
  int64_t t_end = t_begin + tokens_per_chunk;
  if (t_end > N) t_end = N;
  const float* ss = scales + slab * D;
  const float* qb = queries + (slab * q_total + q_first) * D;

#pragma unroll
  for (int k = 0; k < G; k++) {
    const int qi = wave * G + k;
    const bool live = qi < q_count;
    float m = 0.0f;
    if (live)
      for (int64_t d = lane; d < D; d += 64) m = fmaxf(m, fabsf(qb[qi * D + d] * ss[d]));
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    int E = 0;
    (void)frexpf(m, &E);
    const double up = ldexp(1.0, 27 - E);
    double isum = 0.0;  // sum of this lane's I values: integers below 2^53, exact in fp64
    for (int64_t d = lane; d < D; d += 64) {
      int I = 0;
      if (live) I = (int)rint((double)(qb[qi * D + d] * ss[d]) * up);  // |I| <= 2^27
      isum += (double)I;
      const int S = (int)(d >> 7), h = (int)(d >> 5) & 3, mstep = (int)(d >> 4) & 1, c = (int)d & 15;
      unsigned char* p = dig + ((size_t)((S * 2 + mstep) * G + (qi >> 2)) * 64 + 16 * h + 4 * (qi & 3)) * 16 +
                         nibble_pos(c);
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const int pj = ((I + 64) & 127) - 64;
        const int dj = j < 3 ? pj : I;
        p[16 * j] = (unsigned char)(dj & 0xff);
        I = (I - pj) >> 7;
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) isum += __shfl_xor(isum, o);
    if (lane == 0) {
      qscale[qi] = ldexp(1.0, E - 27);
      qsum[qi] = isum;
    }
  }
  __syncthreads();

  const int n = lane & 15, h = lane >> 4;
  const v4i* a_lds = reinterpret_cast<const v4i*>(dig);
  const int64_t prow = D >> 1;  // packed bytes per token
  const uint8_t* cs = packed + slab * N * prow + 16 * h;
  float* os = out + (slab * q_total + q_first) * N;
  const bool vec_store = (N & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0;
  for (int64_t t0 = t_begin + (int64_t)wave * (16 * TU); t0 < t_end; t0 += 4 * 16 * TU) {
    v4i acc[TU][G];
    const uint8_t* row[TU];
#pragma unroll
    for (int u = 0; u < TU; u++) {
      int64_t t = t0 + TU * n + u;  // a lane's four tiles are four consecutive tokens
      if (t >= t_end) t = t_end - 1;
      row[u] = cs + t * prow;
#pragma unroll
      for (int g = 0; g < G; g++) acc[u][g] = v4i{0, 0, 0, 0};
    }
    for (int S = 0; S < dsteps; S++) {
      v4i w[TU];
#pragma unroll
      for (int u = 0; u < TU; u++) w[u] = *reinterpret_cast<const v4i*>(row[u] + 64 * S);
#pragma unroll
      for (int mstep = 0; mstep < 2; mstep++) {
        v4i bv[TU];
#pragma unroll
        for (int u = 0; u < TU; u++) {
          const uint32_t x0 = (uint32_t)w[u][2 * mstep] ^ 0x88888888u, x1 = (uint32_t)w[u][2 * mstep + 1] ^ 0x88888888u;
          bv[u] = v4i{(int)(x0 & 0x0f0f0f0fu), (int)((x0 >> 4) & 0x0f0f0f0fu), (int)(x1 & 0x0f0f0f0fu),
                      (int)((x1 >> 4) & 0x0f0f0f0fu)};
        }
#pragma unroll
        for (int g = 0; g < G; g++) {
          const v4i av = a_lds[((S * 2 + mstep) * G + g) * 64 + lane];
#pragma unroll
          for (int u = 0; u < TU; u++) acc[u][g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bv[u], acc[u][g], 0, 0, 0);
        }
      }
    }
    const int64_t tl = t0 + TU * n;
#pragma unroll
    for (int g = 0; g < G; g++) {
      const int qi = 4 * g + h;
      if (qi >= q_count) continue;
      float v[TU];
#pragma unroll
      for (int u = 0; u < TU; u++) {
        const int64_t S = (int64_t)acc[u][g][0] + (int64_t)acc[u][g][1] * 128 + (int64_t)acc[u][g][2] * 16384 +
                          (int64_t)acc[u][g][3] * 2097152;
        v[u] = (float)(((double)S - 8.0 * qsum[qi]) * qscale[qi]);  // |S| < 2^53: exact until the last product
      }
      float* po = os + qi * N + tl;
      if (vec_store && tl + 4 <= t_end) {
        __builtin_nontemporal_store(f32x4{v[0], v[1], v[2], v[3]}, reinterpret_cast<f32x4*>(po));
      } else {
#pragma unroll
        for (int u = 0; u < TU; u++)
          if (tl + u < t_end) po[u] = v[u];
      }
    }
  }
}

// Any shape: one lane per score, fp32 FMAs in channel order.
__global__ __launch_bounds__(kBlock) void scores_int4_generic_kernel(const float* __restrict__ queries,
                                                                     const uint8_t* __restrict__ packed,
                                                                     const float* __restrict__ scales,
                                                                     float* __restrict__ out, int64_t N, int64_t D,
                                                                     int64_t Q, int64_t total) {
  const int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (i >= total) return;
  const int64_t t = i % N;
  const int64_t j = (i / N) % Q;
  const int64_t slab = i / (N * Q);
  const float* q = queries + (slab * Q + j) * D;
  const uint8_t* c = packed + (slab * N + t) * (D >> 1);
  const float* s = scales + slab * D;
  float acc = 0.0f;
  for (int64_t d = 0; d < D; d += 2) {
    const uint32_t byte = c[d >> 1];
    const int lo = (int)(byte << 28) >> 28, hi = (int)(byte << 24) >> 28;
    acc = fmaf(q[d] * s[d], (float)lo, acc);
    acc = fmaf(q[d + 1] * s[d + 1], (float)hi, acc);
  }
  out[i] = acc;
}

template <int G>
kvq_status launch_int4_g(const float* queries, const uint8_t* packed, const float* scales, float* out, int64_t batch,
                         int64_t N, int64_t D, int64_t q_total, int64_t q_first, int q_count, int cus,
                         hipStream_t stream) {
  // tokens per workgroup: whole passes of 4 waves x 4 tiles, and a walk in proportion to what preparing
  // the digits and their sums costs a workgroup, 1024 G D/128 tokens, but no longer than leaves about two
  // workgroups per compute unit (swept 256..4096 tokens at Q = 1, 4, 8, 16 on [2048 x 4096 x 128],
  // [256 x 4096 x 128], [512 x 4096 x 256]: against 512-2048 tokens for every case, Q = 16 went 0.271 ->
  // 0.246 ms, 0.053 -> 0.033 ms and 0.164 -> 0.092 ms, Q = 1 0.112 -> 0.106 ms on the first)
  const int64_t pass = 4 * 16 * 4;
  int64_t per = (int64_t)1024 * G * (D / 128);
  const int64_t fill = (batch * N + (int64_t)cus * 2 - 1) / ((int64_t)cus * 2);
  if (per > fill) per = fill;
  per = (per + pass - 1) / pass * pass;
  const int64_t chunks = (N + per - 1) / per;
  if (batch * chunks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  const size_t lds_bytes = (size_t)(D / 128) * 2 * G * 1024 + 8 * G * sizeof(double);
  hipLaunchKernelGGL(scores_int4_mfma_kernel<G>, dim3((uint32_t)(batch * chunks)), dim3(kBlock), lds_bytes, stream,
                     queries, packed, scales, out, N, D, q_total, q_first, q_count, (uint32_t)chunks, per);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace

kvq_status launch_scores_from_codes_int4(const float* queries, int64_t Q, const uint8_t* packed, const float* scales,
                                         int64_t batch, int64_t N, int64_t D, float* out, hipStream_t stream) {
  if (D % 128 == 0 && D <= 1024 && aligned(packed, 16)) {
    const DeviceInfo dev = current_device();
    if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
    const int64_t per_pass = D <= 512 ? 16 : 8;
    for (int64_t q0 = 0; q0 < Q; q0 += per_pass) {
      const int qc = (int)(Q - q0 < per_pass ? Q - q0 : per_pass);
      kvq_status s;
      if (qc <= 4) s = launch_int4_g<1>(queries, packed, scales, out, batch, N, D, Q, q0, qc, dev.cus, stream);
      else if (qc <= 8) s = launch_int4_g<2>(queries, packed, scales, out, batch, N, D, Q, q0, qc, dev.cus, stream);
      else s = launch_int4_g<4>(queries, packed, scales, out, batch, N, D, Q, q0, qc, dev.cus, stream);
      if (s != KVQ_OK) return s;
    }
    return KVQ_OK;
  }
  const int64_t total = batch * Q * N;
  const int64_t blocks = (total + kBlock - 1) / kBlock;
  if (blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  hipLaunchKernelGGL(scores_int4_generic_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0, stream, queries, packed,
                     scales, out, N, D, Q, total);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
