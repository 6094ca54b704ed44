// Attention-score error (paper: Introduction, "Attention score error"; Evaluation, "Attention
// Score Error"): the mean over (query, token) of |q.k - q.k_hat|.
//
// This file: the launcher, and the form on the fp32 matrix cores, which takes any shape and alignment.
// Shapes with D a multiple of 128 and aligned pointers take the faster form of kvq_attn_split.hip (the same
// contraction on the bf16 matrix cores, bound by HBM instead of by the matrix rate).
//
// The score difference  q_j . k_t - q_j . k_hat_t = sum_d q_j[d] (k_t[d] - k_hat_t[d])  is a dense
// [tokens x D] . [D x queries] contraction, and e = k - k_hat is exact in fp32 (k_hat is within a
// factor of two of k wherever the code is not 0, and is 0 where it is).  So the contraction runs on
// the fp32 matrix cores (v_mfma_f32_32x32x2_f32), 64 channels at a time, and the 64-channel partial
// dot products are added up in fp64.  With 8 bytes read per key element (5 from codes) and 2 Q
// flops, Q = 64 sits where HBM and the fp32 matrix peak meet (16 flop/B against 157 TFLOP/s over
// 8 TB/s = 20); the fp64 matrix cores, which an earlier version used, make it a compute problem
// twice over (10 flop/B, and fp32 -> fp64 conversions on the vector ALU).
//
// Rounding: within a run of 64 channels every product and every addition is rounded to fp32 once,
// so a score differs from the exact one by at most 65 * 2^-24 * sum_d |q_d e_d|; the additions of the
// runs, the absolute value and the mean are fp64.  The rounding errors are centred, so the mean of
// the absolute scores moves by far less than that bound (measured: below 1e-8 relative on the test
// shapes); the bound itself is what the tests assert per call, next to the 1e-5 bar.
// Preconditions beyond finite inputs: 64-channel partial sums of |q_d e_d| must stay inside the fp32
// range, and products below 2^-126 lose bits (the matrix cores may flush them), which matters only
// for matrices whose scales are themselves near the bottom of the fp32 range.
//
// A workgroup (4 wavefronts) owns 32 tokens x 32*NQ queries and walks D in chunks of 128 channels.
// Per chunk the 256 lanes stage e [32 x 128] and the queries [32*NQ x 128] in LDS as fp32, with
// 512-byte contiguous global reads per row, and wavefront w contracts channels 32w .. 32w+31 of the
// chunk for all tokens and queries: the wavefronts split the channels, not the tokens, so that a
// 32-token tile keeps four wavefronts busy and a [16384 x 8192] matrix gives 512 workgroups, two per
// compute unit.  For a block of 8 channels lane (r = lane % 32, h = lane / 32) reads channels
// 4h .. 4h+3 of token r and of query r of every query tile (one 16-byte LDS read each) and feeds
// four matrix steps; step i contracts channels {i, 4 + i} of the block.  At the end of a tile the
// four wavefronts' fp64 partial scores are added through LDS in a fixed order and the absolute
// values summed.  Tokens, queries and channels outside the matrices are staged as zeros and add |0|.
//
// What shaped the inner loop (measured on this GPU):
//  - a wavefront that streams matrix instructions starves the vector-ALU instructions of the other
//    wavefront on its SIMD completely (a pure v_add stream made no progress next to a matrix stream,
//    then ran at full speed), so vector instructions do not hide behind another wavefront's matrix
//    phase: they add to it.  Hence buffer loads with scalar descriptors (one vector instruction per
//    chunk instead of one or more per load, and no bounds branches), runs that start from a constant
//    zero operand instead of cleared registers, and nothing but the subtraction and the fp64 fold left.
//  - load instructions wait at issue while the compute unit's memory pipeline is full, and a wavefront
//    issues in order: with all 16 loads of a chunk ahead of its matrix steps the matrix cores sat idle
//    for as long as the loads took to issue.  One load after every pair of matrix steps fixed that.
//  - with matrix cores, LDS and HBM all busy the shader clock settles at 1.4-1.7 GHz (shader ticks
//    against the 100 MHz wall clock inside the kernel; a matrix-only loop holds 2.4 GHz and reaches
//    154 TFLOP/s), which is why memory time and matrix time still add up rather than overlap.
#include <type_traits>
#include <utility>

#include "kvq_internal.h"
#include "kvq_reduce.h"

namespace kvq {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTileTok = 32;          // tokens per workgroup: the rows of one 32x32 matrix tile
constexpr int kChunk = 128;           // channels staged per step, 32 per wavefront
constexpr int kPitch = kChunk + 4;    // LDS row pitch in floats: rows 16 bytes askew, so that the
                                      // 16-byte reads of 16 consecutive rows fall into different banks
constexpr int kRunChunks = 2;        // chunks per fp32 accumulation run: 2 * 32 = 64 channels per wavefront
        // chunks per fp32 accumulation run: 2 * 32 = 64 channels per wavefront

struct Quad {
  float v[4];
};

// four consecutive floats p[idx..idx+3] of a row (vector load when VEC), zero where idx + i >= limit or !ok
template <bool VEC, bool NT>
__device__ __forceinline__ Quad load_quad(const float* __restrict__ row, int64_t idx, int64_t limit, bool ok) {
  Quad q;
  if constexpr (VEC) {
    f32x4 t = {0.f, 0.f, 0.f, 0.f};
    if (ok && idx < limit) t = ld<NT>(reinterpret_cast<const f32x4*>(row + idx));
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
    return load_quad<VEC, true>(k_hat + row_off, d, D, ok);
  } else {
    Quad q;
    if constexpr (VEC) {
      uint32_t w = 0;
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
      if (ok && d < D) {
        w = ld<true>(reinterpret_cast<const uint32_t*>(codes + row_off + d));
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

// FAST: D is a multiple of the chunk and every pointer allows 16-byte (codes: 4-byte) access.  Then every
// load is a buffer load: a descriptor per group of 8 rows (base and size in scalar registers, set up once
// per tile) plus one per-lane offset that is the same for all rows and only moves on by 512 bytes per
// chunk, so a chunk's 16 loads cost one vector-ALU instruction, and rows past the end of a matrix come
// back as zeros from the descriptor's range check instead of from branches.  The vector ALU does not
// run while the same SIMD executes a matrix instruction (the co-execution counter of the profiler stays
// at zero for this kernel), so every vector instruction saved is matrix time gained.

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), unrolled at compile time
template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// descriptor of `bytes` bytes at `base` for untyped buffer loads (stride 0; 32-bit data format)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_buffer(const void* base, int64_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
template <bool NT>
__device__ __forceinline__ f32x4 buffer_ld16(__amdgpu_buffer_rsrc_t rsrc, uint32_t offset) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)offset, 0, NT ? 2 : 0);
  f32x4 f;
  __builtin_memcpy(&f, &v, 16);
  return f;
}

template <int NQ, bool VEC, bool FROM_CODES, bool FAST>
__global__ __launch_bounds__(kBlock, 2) void attn_score_kernel(const float* __restrict__ queries, int64_t Q,
                                                               const float* __restrict__ k,
                                                               const float* __restrict__ k_hat,
                                                               const int8_t* __restrict__ codes,
                                                               const float* __restrict__ scales, int64_t N,
                                                               int64_t D, uint32_t qchunks, uint32_t tiles,
                                                               double* __restrict__ sums) {
  static_assert(!FAST || VEC, "buffer loads are vector loads");
  constexpr int QR = 32 * NQ;                  // query rows staged per chunk
  constexpr int ROWS_PER_PASS = kBlock / (kChunk / 4);  // 8 rows of 32 sixteen-byte pieces per fill pass
  constexpr int KP = kTileTok / ROWS_PER_PASS; // fill passes for the token rows
  constexpr int QP = QR / ROWS_PER_PASS;       // and for the query rows
  // one buffer, used as [32 + QR][kPitch] floats while a tile is contracted and as [3][16*NQ][64]
  // doubles when the wavefronts' partial scores meet
  __shared__ __align__(16) float lds[(kTileTok + QR) * kPitch];
  static_assert(sizeof(float) * (kTileTok + QR) * kPitch >= sizeof(double) * 3 * 16 * NQ * 64, "combine area");
  float* const e_s = lds;
  float* const q_s = lds + kTileTok * kPitch;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31;    // row of the 32-row operand tile: a token (A) or a query (B)
  const int h = lane >> 5;    // which half of an 8-channel block this lane supplies
  const int frow = tid >> 5;  // fill role: row within a pass, and which 16-byte piece of the chunk
  const int fcol = (tid & 31) * 4;
  // byte offset of this lane's piece from the first row of a fill pass (the host checked that 8 rows fit 32 bits)
  const uint32_t lane_off = (uint32_t)(((int64_t)frow * D + fcol) * 4);
  const int64_t nchunks = (D + kChunk - 1) / kChunk;
  double total = 0.0;

  for (uint32_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
    const int64_t q0 = (int64_t)(tile % qchunks) * QR;
    const int64_t t0 = (int64_t)(tile / qchunks) * kTileTok;
    f32x16 acc[NQ];
    double acc64[NQ][16];
#pragma unroll
    for (int n = 0; n < NQ; n++)
#pragma unroll
      for (int i = 0; i < 16; i++) acc64[n][i] = 0.0;

    // descriptors of the tile's row groups: 8 rows each, cut off where the matrix ends
    __amdgpu_buffer_rsrc_t kr[KP], hr[KP], qr[QP], sr;
    if constexpr (FAST) {
      auto rows_left = [](int64_t have, int64_t first) {
        const int64_t n = have - first;
        return n < 0 ? (int64_t)0 : (n > ROWS_PER_PASS ? (int64_t)ROWS_PER_PASS : n);
      };
#pragma unroll
      for (int p = 0; p < KP; p++) {
        const int64_t row = t0 + p * ROWS_PER_PASS, rows = rows_left(N, row);
        const int64_t first = rows ? row : 0;  // keep the base inside the matrix when nothing is left
        kr[p] = raw_buffer(k + first * D, rows * D * 4);
        if constexpr (FROM_CODES) hr[p] = raw_buffer(codes + first * D, rows * D);
        else hr[p] = raw_buffer(k_hat + first * D, rows * D * 4);
      }
#pragma unroll
      for (int p = 0; p < QP; p++) {
        const int64_t row = q0 + p * ROWS_PER_PASS, rows = rows_left(Q, row);
        qr[p] = raw_buffer(queries + (rows ? row : 0) * D, rows * D * 4);
      }
      if constexpr (FROM_CODES) sr = raw_buffer(scales, D * 4);
    }

    f32x4 kv[KP], hv[KP], qv[QP], sv;
    uint32_t wv[KP];
    // One load of the next chunk; slot 0 .. KP-1: k, KP .. 2KP-1: k_hat (or codes; the last of them brings the
    // scales along), then the queries.  They are issued one at a time between the matrix steps of the
    // chunk before: a wavefront issues in order, a load waits at issue while the memory pipeline of the
    // compute unit is full, and only what was issued before it keeps the matrix cores busy meanwhile.
    auto fetch_slot = [&](uint32_t voff, auto slot_tag) {
      constexpr int SLOT = decltype(slot_tag)::value;
      if constexpr (SLOT < KP) {
        kv[SLOT] = buffer_ld16<true>(kr[SLOT], voff);
      } else if constexpr (SLOT < 2 * KP) {
        constexpr int P = SLOT - KP;
        if constexpr (FROM_CODES) {
          wv[P] = __builtin_amdgcn_raw_buffer_load_b32(hr[P], (int)(voff >> 2), 0, 2);
          if constexpr (P == KP - 1) sv = buffer_ld16<false>(sr, voff - lane_off + (uint32_t)fcol * 4);
        } else {
          hv[P] = buffer_ld16<true>(hr[P], voff);
        }
      } else if constexpr (SLOT < 2 * KP + QP) {
        qv[SLOT - 2 * KP] = buffer_ld16<false>(qr[SLOT - 2 * KP], voff);
      }
    };
    // all loads of a chunk at once: first chunk of a tile, and every chunk of the checked (not FAST) form
    auto fetch_all = [&](int64_t chunk) {
      if constexpr (FAST) {
        const uint32_t voff = lane_off + (uint32_t)chunk * (kChunk * 4);
        static_for<2 * KP + QP>([&](auto slot_tag) { fetch_slot(voff, slot_tag); });
      } else {
        const int64_t d = chunk * kChunk + fcol;
#pragma unroll
        for (int p = 0; p < KP; p++) {
          const int64_t tok = t0 + frow + p * ROWS_PER_PASS;
          const Quad a = load_quad<VEC, true>(k + tok * D, d, D, tok < N);
          const Quad b = load_khat<VEC, FROM_CODES>(k_hat, codes, scales, tok * D, d, D, tok < N);
          kv[p] = f32x4{a.v[0], a.v[1], a.v[2], a.v[3]};
          hv[p] = f32x4{b.v[0], b.v[1], b.v[2], b.v[3]};
        }
#pragma unroll
        for (int p = 0; p < QP; p++) {
          const int64_t qi = q0 + frow + p * ROWS_PER_PASS;
          const Quad a = load_quad<VEC, false>(queries + qi * D, d, D, qi < Q);
          qv[p] = f32x4{a.v[0], a.v[1], a.v[2], a.v[3]};
        }
      }
    };
    auto stage = [&]() {
      if constexpr (FAST && FROM_CODES) {
#pragma unroll
        for (int p = 0; p < KP; p++)
#pragma unroll
          for (int i = 0; i < 4; i++) hv[p][i] = (float)((int)(wv[p] << (24 - 8 * i)) >> 24) * sv[i];
      }
#pragma unroll
      for (int p = 0; p < KP; p++)
        *reinterpret_cast<f32x4*>(e_s + (frow + p * ROWS_PER_PASS) * kPitch + fcol) = kv[p] - hv[p];
#pragma unroll
      for (int p = 0; p < QP; p++)
        *reinterpret_cast<f32x4*>(q_s + (frow + p * ROWS_PER_PASS) * kPitch + fcol) = qv[p];
    };

    // Workgroups start their sweep over the channels at different chunks, so that they do not all ask
    // for the same lines of the queries at the same moment (the order of the chunks does not matter to
    // the sum).
    int64_t chunk = (int64_t)((tile / qchunks) * 5u % (uint32_t)nchunks);
    fetch_all(chunk);
    __syncthreads();  // the previous tile's partial scores have been read out of the buffer
    stage();
    __syncthreads();
    int in_run = 0;
    const float* ep = e_s + r * kPitch + 32 * wave + 4 * h;
    const float* qp = q_s + r * kPitch + 32 * wave + 4 * h;
    for (int64_t done = 1; done <= nchunks; done++) {
      const bool more = done < nchunks;
      chunk = chunk + 1 == nchunks ? 0 : chunk + 1;
      const uint32_t voff = lane_off + (uint32_t)chunk * (kChunk * 4);
      if constexpr (!FAST) {
        if (more) fetch_all(chunk);
      }
      // operands of block m + 1 are read from LDS before the matrix steps of block m are issued, and one
      // load of the next chunk goes out after every pair of matrix steps
      f32x4 a = *reinterpret_cast<const f32x4*>(ep);
      f32x4 b[NQ];
#pragma unroll
      for (int n = 0; n < NQ; n++) b[n] = *reinterpret_cast<const f32x4*>(qp + 32 * n * kPitch);
      auto block = [&](auto m_tag) {
        constexpr int m = decltype(m_tag)::value;
        f32x4 a_n = a, b_n[NQ];
#pragma unroll
        for (int n = 0; n < NQ; n++) b_n[n] = b[n];
        if constexpr (m + 1 < 4) {
          a_n = *reinterpret_cast<const f32x4*>(ep + 8 * (m + 1));
#pragma unroll
          for (int n = 0; n < NQ; n++) b_n[n] = *reinterpret_cast<const f32x4*>(qp + 32 * n * kPitch + 8 * (m + 1));
        }
        static_for<4>([&](auto i_tag) {
          constexpr int I = decltype(i_tag)::value;
          if (m == 0 && I == 0 && in_run == 0) {
            // a run starts from zero: the constant operand saves clearing 16 registers per tile
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int n = 0; n < NQ; n++) acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[I], b[n][I], zero, 0, 0, 0);
          } else {
#pragma unroll
            for (int n = 0; n < NQ; n++) acc[n] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[I], b[n][I], acc[n], 0, 0, 0);
          }
          if constexpr (FAST) {
            __builtin_amdgcn_sched_barrier(0);
            // (after the last chunk this fetches the tile's first chunk once more, unused: cheaper than
            // a branch around every load)
            fetch_slot(voff, std::integral_constant<int, 4 * m + I>{});
            __builtin_amdgcn_sched_barrier(0);
          }
        });
        a = a_n;
#pragma unroll
        for (int n = 0; n < NQ; n++) b[n] = b_n[n];
      };
      block(std::integral_constant<int, 0>{});
      block(std::integral_constant<int, 1>{});
      block(std::integral_constant<int, 2>{});
      block(std::integral_constant<int, 3>{});
      static_assert(2 * KP + QP <= 16, "one load slot per pair of matrix steps");
      if (++in_run == kRunChunks || !more) {
        // the run's fp32 sums join the fp64 totals
#pragma unroll
        for (int n = 0; n < NQ; n++)
#pragma unroll
          for (int i = 0; i < 16; i++) acc64[n][i] += (double)acc[n][i];
        in_run = 0;
      }
      __syncthreads();  // every wavefront has read this chunk
      if (more) {
        stage();
        __syncthreads();
      }
    }

    // the four wavefronts hold the partial scores of their quarter of the channels
    double* const comb = reinterpret_cast<double*>(lds);
    if (wave > 0) {
#pragma unroll
      for (int n = 0; n < NQ; n++)
#pragma unroll
        for (int i = 0; i < 16; i++) comb[(((wave - 1) * NQ + n) * 16 + i) * 64 + lane] = acc64[n][i];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int n = 0; n < NQ; n++)
#pragma unroll
        for (int i = 0; i < 16; i++) {
          double s = acc64[n][i];
#pragma unroll
          for (int w = 0; w < 3; w++) s += comb[((w * NQ + n) * 16 + i) * 64 + lane];
          total += fabs(s);
        }
    }
  }
  float unused = 0.0f;
  __syncthreads();
  block_reduce(total, unused);
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

kvq_status launch_attn_score_error(const float* queries, int64_t Q, const float* k, const float* k_hat,
                                   const int8_t* codes, const float* scales, int64_t N, int64_t D,
                                   double* mean_abs_out, hipStream_t stream) {
  Workspace ws;
  if (kvq_status s = get_workspace(stream, &ws)) return s;
  const int NQ = Q > 32 ? 2 : 1;  // query tiles of 32 per workgroup
  const int64_t qchunks = (Q + 32 * NQ - 1) / (32 * NQ);
  const int64_t ttiles = (N + kTileTok - 1) / kTileTok;
  if (qchunks > INT32_MAX / 2 || ttiles > INT32_MAX / qchunks) return KVQ_ERR_OVERFLOW;
  const int64_t tiles = qchunks * ttiles;
  const int64_t blocks = tiles < kMaxPartials ? tiles : kMaxPartials;
  const bool from_codes = k_hat == nullptr;
  bool vec = D % 4 == 0 && aligned(queries, 16) && aligned(k, 16);
  vec = vec && (from_codes ? (aligned(codes, 4) && aligned(scales, 16)) : aligned(k_hat, 16));
  // unchecked loads: whole chunks, vector access, and per-lane byte offsets (8 rows at most) within 32 bits
  const bool fast = vec && D % kChunk == 0 && D <= ((int64_t)1 << 26);
  if (fast && attn_split_applicable(Q, D) && options().attn_form != 1) {
    int nblocks = 0;
    if (kvq_status s = launch_attn_split(queries, Q, k, k_hat, codes, scales, N, D, ws, &nblocks, stream)) return s;
    return launch_fold_partials(ws.sums, nullptr, nblocks, (double)Q * (double)N, mean_abs_out, nullptr, stream);
  }
  const dim3 grid((uint32_t)blocks), block(kBlock);
#define KVQ_LAUNCH_AS(NQ_, VEC_, FC_, FAST_)                                                                 \
  hipLaunchKernelGGL((attn_score_kernel<NQ_, VEC_, FC_, FAST_>), grid, block, 0, stream, queries, Q, k, k_hat, \
                     codes, scales, N, D, (uint32_t)qchunks, (uint32_t)tiles, ws.sums)
#define KVQ_PICK_AS(NQ_)                                               \
  do {                                                                 \
    if (fast && from_codes) KVQ_LAUNCH_AS(NQ_, true, true, true);      \
    else if (fast) KVQ_LAUNCH_AS(NQ_, true, false, true);              \
    else if (vec && from_codes) KVQ_LAUNCH_AS(NQ_, true, true, false); \
    else if (vec) KVQ_LAUNCH_AS(NQ_, true, false, false);              \
    else if (from_codes) KVQ_LAUNCH_AS(NQ_, false, true, false);       \
    else KVQ_LAUNCH_AS(NQ_, false, false, false);                      \
  } while (0)
  if (NQ == 2) KVQ_PICK_AS(2);
  else KVQ_PICK_AS(1);
#undef KVQ_PICK_AS
#undef KVQ_LAUNCH_AS
  KVQ_HIP(hipGetLastError());
  return launch_fold_partials(ws.sums, nullptr, (int)blocks, (double)Q * (double)N, mean_abs_out, nullptr, stream);
}

}  // namespace kvq
