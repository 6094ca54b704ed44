// Attention scores from the quantized cache on the matrix cores, for several queries per head
// (paper: Background, Eq. (attention) with the reconstruction of Eq. (dequant_op); "Future Work").
//
//   scores[b,j,t] = sum_d (q[b,j,d] * s[b,d]) * code[b,t,d]
//
// The codes are int8 already, so they go from HBM straight into the B operand of the int8 MFMA
// (v_mfma_i32_16x16x64_i8): no per-code vector ALU work at all.  The folded queries qs = q * s
// (fp32) are turned, once per workgroup, into 28-bit fixed point relative to the largest |qs| of
// their query and cut into four balanced base-128 digits, each an int8:
//   qs[d] ~ 2^(E-27) * I[d],   I[d] = p0 + 128 p1 + 128^2 p2 + 128^3 p3,  |I| <= 2^27, p in [-64, 64]
// The A operand holds 16 rows = 4 queries x 4 digits; the int32 accumulators are exact, the four
// digit sums of a query land in the four accumulator registers of one lane and are recombined in
// int64, scaled by 2^(E-27) in fp64 and rounded once to fp32.  The only approximation is the
// fixed-point step: |qs[d] - 2^(E-27) I[d]| <= 2^(E-28) <= 2^-27 max_d |qs[d]|.  The result does not
// depend on the launch shape or on the order of accumulation.
//
// Operand layout of the 16x16x64 instruction (wave64): lane = 16 h + i; A: row i, B: column i,
// both holding 16 consecutive k of k-group h; C: column i, rows 4 h + r in register r.  A and B use
// the same k numbering, so all that matters is that both are filled from the same channels:
// byte b of k-group h in step s is channel 64 s + 16 h + b -- a lane's B operand is one 16-byte
// load from its token's row, and the 4 lanes of a token cover 64 contiguous bytes.
#include "kvq_internal.h"

namespace kvq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));


// G = groups of 4 queries handled per pass over the codes.  STEPS = D / 64 when that is 1, 2 or 4
// (all loads of a tile group are then issued together, the loads that share a cache line next to
// each other), 0 for any other D (a runtime loop over the steps).  TU = token tiles in flight.
template <int G, int STEPS, int TU, bool NT, bool NT_OUT>
__global__ __launch_bounds__(kBlock) void scores_mfma_kernel(const float* __restrict__ queries,
                                                             const int8_t* __restrict__ codes,
                                                             const float* __restrict__ scales,
                                                             float* __restrict__ out, int64_t N, int64_t D,
                                                             int64_t q_total, int64_t q_first, int q_count,
                                                             uint32_t chunks, int64_t tokens_per_chunk) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int steps = (int)(D >> 6);
  // [steps][G][64 lanes][16 bytes] digits, then one fp64 factor 2^(E-27) per query
  unsigned char* dig = lds;
  double* qscale = reinterpret_cast<double*>(lds + (size_t)steps * G * 1024);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int64_t slab = blockIdx.x / chunks;
  const int64_t t_begin = (int64_t)(blockIdx.x % chunks) * tokens_per_chunk;
  int64_t t_end = t_begin + tokens_per_chunk;
  if (t_end > N) t_end = N;
  const float* ss = scales + slab * D;
  const float* qb = queries + (slab * q_total + q_first) * D;

  // ---- fold, find each query's range, cut into digits: wavefront w prepares queries w*G .. w*G+G-1 ----
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
    (void)frexpf(m, &E);  // m = f * 2^E with f in [0.5, 1): |qs| < 2^E; E = 0 for m == 0
    const double up = ldexp(1.0, 27 - E);
    if (lane == 0) qscale[qi] = ldexp(1.0, E - 27);
    for (int64_t d = lane; d < D; d += 64) {
      int I = 0;
      if (live) I = (int)rint((double)(qb[qi * D + d] * ss[d]) * up);  // |I| <= 2^27
      const int s = (int)(d >> 6), h = (int)(d >> 4) & 3, b = (int)d & 15;
      unsigned char* p = dig + ((size_t)(s * G + (qi >> 2)) * 64 + 16 * h + 4 * (qi & 3)) * 16 + b;
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const int pj = ((I + 64) & 127) - 64;  // balanced digit in [-64, 63]; the last one is what is left
        const int dj = j < 3 ? pj : I;
        p[16 * j] = (unsigned char)(dj & 0xff);
        I = (I - pj) >> 7;
      }
    }
  }
  __syncthreads();

  // ---- the codes ----
  const int n = lane & 15, h = lane >> 4;
  const v4i* a_lds = reinterpret_cast<const v4i*>(dig);
  const int8_t* cs = codes + slab * N * D + 16 * h;
  float* os = out + (slab * q_total + q_first) * N;
  // A wavefront works on 16 * TU consecutive tokens at a time.  Rows longer than 64 bytes: column n of
  // tile u is token t0 + TU * n + u, so a lane ends up with TU consecutive tokens of a query and stores
  // them as one vector.  64-byte rows: column n of tile u is token t0 + 16 u + n, which makes every
  // load instruction one contiguous KiB (measured 15 % faster there than the interleaved form).
  constexpr bool kInterleave = STEPS != 1;
  constexpr int kTokStride = kInterleave ? TU : 1;   // between the columns of a tile
  constexpr int kTileStride = kInterleave ? 1 : 16;  // between the tiles of a lane
  const bool vec_store = kInterleave && TU == 4 && (N & 3) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0;
  for (int64_t t0 = t_begin + (int64_t)wave * (16 * TU); t0 < t_end; t0 += 4 * 16 * TU) {
    v4i acc[TU][G];
    const int8_t* row[TU];
#pragma unroll
    for (int u = 0; u < TU; u++) {
      int64_t t = t0 + kTokStride * n + kTileStride * u;
      if (t >= t_end) t = t_end - 1;  // clamp the load; the store below is skipped
      row[u] = cs + t * D;
#pragma unroll
      for (int g = 0; g < G; g++) acc[u][g] = v4i{0, 0, 0, 0};
    }
    if constexpr (STEPS > 0) {
      v4i bv[TU][STEPS];
#pragma unroll
      for (int u = 0; u < TU; u++)
#pragma unroll
        for (int s = 0; s < STEPS; s++) bv[u][s] = ld<NT>(reinterpret_cast<const v4i*>(row[u] + 64 * s));
#pragma unroll
      for (int s = 0; s < STEPS; s++)
#pragma unroll
        for (int g = 0; g < G; g++) {
          const v4i av = a_lds[(s * G + g) * 64 + lane];
#pragma unroll
          for (int u = 0; u < TU; u++)
            acc[u][g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bv[u][s], acc[u][g], 0, 0, 0);
        }
    } else {
      // runtime number of steps: four at a time, so that every visit of a token's row fetches 256
      // contiguous bytes (tokens of a tile lie in different DRAM pages once rows are long)
      int s = 0;
      for (; s + 4 <= steps; s += 4) {
        v4i bv[TU][4];
#pragma unroll
        for (int u = 0; u < TU; u++)
#pragma unroll
          for (int k = 0; k < 4; k++) bv[u][k] = ld<NT>(reinterpret_cast<const v4i*>(row[u] + 64 * (s + k)));
#pragma unroll
        for (int k = 0; k < 4; k++)
#pragma unroll
          for (int g = 0; g < G; g++) {
            const v4i av = a_lds[((s + k) * G + g) * 64 + lane];
#pragma unroll
            for (int u = 0; u < TU; u++)
              acc[u][g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bv[u][k], acc[u][g], 0, 0, 0);
          }
      }
      for (; s < steps; s++) {
        v4i bv[TU];
#pragma unroll
        for (int u = 0; u < TU; u++) bv[u] = ld<NT>(reinterpret_cast<const v4i*>(row[u] + 64 * s));
#pragma unroll
        for (int g = 0; g < G; g++) {
          const v4i av = a_lds[(s * G + g) * 64 + lane];
#pragma unroll
          for (int u = 0; u < TU; u++) acc[u][g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bv[u], acc[u][g], 0, 0, 0);
        }
      }
    }
    const int64_t tl = t0 + kTokStride * n;  // first of this lane's TU tokens
#pragma unroll
    for (int g = 0; g < G; g++) {
      const int qi = 4 * g + h;  // rows 4 h + r of the tile: query h of the group, digit r
      if (qi >= q_count) continue;
      float v[TU];
#pragma unroll
      for (int u = 0; u < TU; u++) {
        const int64_t S = (int64_t)acc[u][g][0] + (int64_t)acc[u][g][1] * 128 + (int64_t)acc[u][g][2] * 16384 +
                          (int64_t)acc[u][g][3] * 2097152;
        v[u] = (float)((double)S * qscale[qi]);
      }
      float* po = os + qi * N + tl;
      if constexpr (TU == 4) {
        if (vec_store && tl + 4 <= t_end) {
          st<NT_OUT>(reinterpret_cast<f32x4*>(po), f32x4{v[0], v[1], v[2], v[3]});
          continue;
        }
      }
#pragma unroll
      for (int u = 0; u < TU; u++)
        if (tl + kTileStride * u < t_end) st<NT_OUT>(po + kTileStride * u, v[u]);
    }
  }
}

// Rows wider than 1024 channels (up to 8192): the digits of 4 G queries for the whole row resident in
// 128 KiB of LDS -- G = 1 group of four queries per pass over the codes for rows of up to 8192 channels,
// 2 up to 4096, 4 up to 2048 -- one workgroup of 16 wavefronts per compute unit.  Wavefront w prepares
// quarter w / 4 of query w % 4 of every group; the token loop is the one above with a runtime number of
// steps.
constexpr int kWideBlock = 1024;
constexpr int kWideMaxD = 8192;

template <int G>
__global__ __launch_bounds__(kWideBlock) void scores_mfma_wide_kernel(const float* __restrict__ queries,
                                                                      const int8_t* __restrict__ codes,
                                                                      const float* __restrict__ scales,
                                                                      float* __restrict__ out, int64_t N, int64_t D,
                                                                      int64_t q_total, int64_t q_first, int q_count,
                                                                      uint32_t chunks, int64_t tokens_per_chunk) {
  __shared__ __align__(16) unsigned char dig[kWideMaxD * 16];  // [steps][G][64 lanes][16 bytes], G * D <= 8192
  __shared__ double qscale[4 * G];
  __shared__ float red[G][16];
  const int steps = (int)(D >> 6);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int64_t slab = blockIdx.x / chunks;
  const int64_t t_begin = (int64_t)(blockIdx.x % chunks) * tokens_per_chunk;
  int64_t t_end = t_begin + tokens_per_chunk;
  if (t_end > N) t_end = N;
  const float* ss = scales + slab * D;
  const float* qb = queries + (slab * q_total + q_first) * D;

  {
    const int64_t d_lo = (int64_t)(wave >> 2) * (D >> 2), d_hi = d_lo + (D >> 2);
    float m[G];
#pragma unroll
    for (int g = 0; g < G; g++) {
      const int qi = 4 * g + (wave & 3);
      m[g] = 0.0f;
      if (qi < q_count)
        for (int64_t d = d_lo + lane; d < d_hi; d += 64) m[g] = fmaxf(m[g], fabsf(qb[qi * D + d] * ss[d]));
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) m[g] = fmaxf(m[g], __shfl_xor(m[g], o));
      if (lane == 0) red[g][wave] = m[g];
    }
    __syncthreads();
#pragma unroll
    for (int g = 0; g < G; g++) {
      const int q4 = wave & 3, qi = 4 * g + q4;
      const bool live = qi < q_count;
      const float mm = fmaxf(fmaxf(red[g][q4], red[g][q4 + 4]), fmaxf(red[g][q4 + 8], red[g][q4 + 12]));
      int E = 0;
      (void)frexpf(mm, &E);
      const double up = ldexp(1.0, 27 - E);
      if (wave < 4 && lane == 0) qscale[qi] = ldexp(1.0, E - 27);
      for (int64_t d = d_lo + lane; d < d_hi; d += 64) {
        int I = 0;
        if (live) I = (int)rint((double)(qb[qi * D + d] * ss[d]) * up);
        const int s = (int)(d >> 6), h = (int)(d >> 4) & 3, b = (int)d & 15;
        unsigned char* p = dig + ((size_t)(s * G + g) * 64 + 16 * h + 4 * q4) * 16 + b;
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const int pj = ((I + 64) & 127) - 64;
          const int dj = j < 3 ? pj : I;
          p[16 * j] = (unsigned char)(dj & 0xff);
          I = (I - pj) >> 7;
        }
      }
    }
  }
  __syncthreads();

  const int n = lane & 15, h = lane >> 4;
  const v4i* a_lds = reinterpret_cast<const v4i*>(dig);
  const int8_t* cs = codes + slab * N * D + 16 * h;
  float* os = out + (slab * q_total + q_first) * N;
  const bool vec_store = (N & 1) == 0 && (reinterpret_cast<uintptr_t>(out) & 7) == 0;
  // A wavefront takes TW tiles of 16 tokens and walks the row SU steps (SU * 64 channels) at a time, so
  // that every visit of a token's row fetches SU * 64 contiguous bytes: with rows of several KiB the
  // tokens of a tile lie in different DRAM pages, and short visits would reopen them over and over.
  constexpr int TW = 2, SU = 4;
  for (int64_t t0 = t_begin + (int64_t)wave * (16 * TW); t0 < t_end; t0 += (kWideBlock / 64) * 16 * TW) {
    v4i acc[TW][G];
    const int8_t* row[TW];
#pragma unroll
    for (int u = 0; u < TW; u++) {
      int64_t t = t0 + TW * n + u;  // a lane's tiles are consecutive tokens
      if (t >= t_end) t = t_end - 1;
      row[u] = cs + t * D;
#pragma unroll
      for (int g = 0; g < G; g++) acc[u][g] = v4i{0, 0, 0, 0};
    }
    for (int s = 0; s < steps; s += SU) {  // steps is a multiple of 4: D % 256 == 0 on this path
      v4i bv[TW][SU];
#pragma unroll
      for (int u = 0; u < TW; u++)
#pragma unroll
        for (int k = 0; k < SU; k++) bv[u][k] = *reinterpret_cast<const v4i*>(row[u] + 64 * (s + k));
#pragma unroll
      for (int k = 0; k < SU; k++)
#pragma unroll
        for (int g = 0; g < G; g++) {
          const v4i av = a_lds[((s + k) * G + g) * 64 + lane];
#pragma unroll
          for (int u = 0; u < TW; u++)
            acc[u][g] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av, bv[u][k], acc[u][g], 0, 0, 0);
        }
    }
    const int64_t tl = t0 + TW * n;
#pragma unroll
    for (int g = 0; g < G; g++) {
      const int qi = 4 * g + h;
      if (qi >= q_count) continue;
      float v[TW];
#pragma unroll
      for (int u = 0; u < TW; u++) {
        const int64_t S = (int64_t)acc[u][g][0] + (int64_t)acc[u][g][1] * 128 + (int64_t)acc[u][g][2] * 16384 +
                          (int64_t)acc[u][g][3] * 2097152;
        v[u] = (float)((double)S * qscale[qi]);
      }
      float* po = os + qi * N + tl;
      if (vec_store && tl + 2 <= t_end) {
        __builtin_nontemporal_store(f32x2{v[0], v[1]}, reinterpret_cast<f32x2*>(po));
      } else {
#pragma unroll
        for (int u = 0; u < TW; u++)
          if (tl + u < t_end) po[u] = v[u];
      }
    }
  }
}

template <int G, int STEPS, int TU>
kvq_status launch_g(const float* queries, const int8_t* codes, const float* scales, float* out, int64_t batch,
                    int64_t N, int64_t D, int64_t q_total, int64_t q_first, int q_count, int cus, size_t lds_bytes,
                    hipStream_t stream) {
  // tokens per workgroup: whole passes of 4 waves x TU tiles.  Preparing the digits costs a workgroup
  // time in proportion to queries x channels, so its walk grows with that: 256 G D/64 tokens for rows of
  // 64-256 channels (swept 256..8192 tokens on [2048 x 4096 x 128], [4096 x 4096 x 64], [512 x 4096 x
  // 256] at Q = 4, 8, 16: within 2 % of the best of each, up to 14 % better than one size for all), but
  // no longer than leaves about 4 workgroups per compute unit.
  const int64_t pass = 4 * 16 * TU;
  int64_t per;
  if (STEPS > 0) {
    per = (int64_t)256 * G * STEPS;
    const int64_t fill = (batch * N + (int64_t)cus * 4 - 1) / ((int64_t)cus * 4);
    if (per > fill) per = fill;
    per = (per + pass - 1) / pass * pass;
  } else {
    const int64_t want = (int64_t)cus * 16;
    per = (batch * N + want - 1) / want;
    per = (per + pass - 1) / pass * pass;
    if (per < 512) per = 512;
  }
  const int64_t chunks = (N + per - 1) / per;
  if (batch * chunks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  const dim3 grid((uint32_t)(batch * chunks)), block(kBlock);
  // nontemporal loads only where one load instruction covers whole cache lines (64-byte rows): with longer
  // rows a line is shared by consecutive instructions and must stay in the first-level cache between them
  if (options().nontemporal)
    hipLaunchKernelGGL((scores_mfma_kernel<G, STEPS, TU, STEPS == 1, true>), grid, block, lds_bytes, stream, queries,
                       codes, scales, out, N, D, q_total, q_first, q_count, (uint32_t)chunks, per);
  else
    hipLaunchKernelGGL((scores_mfma_kernel<G, STEPS, TU, false, false>), grid, block, lds_bytes, stream, queries,
                       codes, scales, out, N, D, q_total, q_first, q_count, (uint32_t)chunks, per);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

template <int G>
kvq_status launch_steps(const float* queries, const int8_t* codes, const float* scales, float* out, int64_t batch,
                        int64_t N, int64_t D, int64_t q_total, int64_t q_first, int q_count, int cus,
                        size_t lds_bytes, hipStream_t stream) {
  if (D == 64)
    return launch_g<G, 1, 4>(queries, codes, scales, out, batch, N, D, q_total, q_first, q_count, cus, lds_bytes, stream);
  if (D == 128)
    return launch_g<G, 2, 4>(queries, codes, scales, out, batch, N, D, q_total, q_first, q_count, cus, lds_bytes, stream);
  if (D == 256)
    return launch_g<G, 4, 2>(queries, codes, scales, out, batch, N, D, q_total, q_first, q_count, cus, lds_bytes, stream);
  return launch_g<G, 0, 2>(queries, codes, scales, out, batch, N, D, q_total, q_first, q_count, cus, lds_bytes, stream);
}

}  // namespace

bool scores_mfma_applicable(const float* queries, int64_t Q, const int8_t* codes, const float* scales, int64_t D) {
  (void)queries;
  (void)scales;
  // 16-byte code loads of whole 64-channel steps; digits of 8-16 queries in 32 KiB of LDS up to 1024
  // channels, of 4 / 8 / 16 queries in 128 KiB up to 8192 / 4096 / 2048 channels (quarters of a row must be whole
  // 16-byte pieces)
  return Q >= 3 && D % 64 == 0 && (D <= 1024 || (D % 256 == 0 && D <= kWideMaxD)) && aligned(codes, 16);
}

kvq_status launch_scores_mfma(const float* queries, int64_t Q, const int8_t* codes, const float* scales,
                              int64_t batch, int64_t N, int64_t D, float* out, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  if (D > 1024) {
    // one workgroup per compute unit; whole passes of 16 wavefronts x 4 tiles of 16 tokens
    const int64_t pass = (kWideBlock / 64) * 16 * 2;
    int64_t per = (batch * N + dev.cus - 1) / dev.cus;
    per = (per + pass - 1) / pass * pass;
    const int64_t chunks = (N + per - 1) / per;
    if (batch * chunks > INT32_MAX) return KVQ_ERR_OVERFLOW;
    // groups of four queries per pass: as many as keep the digits of a whole row within the 128 KiB
    const int groups = D <= 2048 ? 4 : D <= 4096 ? 2 : 1;
    const dim3 grid((uint32_t)(batch * chunks)), block(kWideBlock);
    for (int64_t q0 = 0; q0 < Q; q0 += 4 * groups) {
      const int qc = (int)(Q - q0 < 4 * groups ? Q - q0 : 4 * groups);
      if (qc > 8)
        hipLaunchKernelGGL(scores_mfma_wide_kernel<4>, grid, block, 0, stream, queries, codes, scales, out, N, D, Q, q0,
                           qc, (uint32_t)chunks, per);
      else if (qc > 4)
        hipLaunchKernelGGL(scores_mfma_wide_kernel<2>, grid, block, 0, stream, queries, codes, scales, out, N, D, Q, q0,
                           qc, (uint32_t)chunks, per);
      else
        hipLaunchKernelGGL(scores_mfma_wide_kernel<1>, grid, block, 0, stream, queries, codes, scales, out, N, D, Q, q0,
                           qc, (uint32_t)chunks, per);
      KVQ_HIP(hipGetLastError());
    }
    return KVQ_OK;
  }
  const int64_t per_pass = D <= 512 ? 16 : 8;  // queries per pass over the codes (digits within 32 KiB of LDS)
  for (int64_t q0 = 0; q0 < Q; q0 += per_pass) {
    const int qc = (int)(Q - q0 < per_pass ? Q - q0 : per_pass);
    const int G = qc <= 4 ? 1 : qc <= 8 ? 2 : 4;
    const size_t lds_bytes = (size_t)(D / 64) * G * 1024 + 4 * G * sizeof(double);
    kvq_status s;
    if (G == 1) s = launch_steps<1>(queries, codes, scales, out, batch, N, D, Q, q0, qc, dev.cus, lds_bytes, stream);
    else if (G == 2) s = launch_steps<2>(queries, codes, scales, out, batch, N, D, Q, q0, qc, dev.cus, lds_bytes, stream);
    else s = launch_steps<4>(queries, codes, scales, out, batch, N, D, Q, q0, qc, dev.cus, lds_bytes, stream);
    if (s != KVQ_OK) return s;
  }
  return KVQ_OK;
}

}  // namespace kvq
