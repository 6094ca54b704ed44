// Attention-score error (paper: Introduction, "Attention score error"; Evaluation, "Attention
// Score Error") on the bf16 matrix cores, for shapes whose rows allow unchecked 16-byte access.
//
// The contraction  sum_d q_j[d] e_t[d]  with e = k - k_hat (exact in fp32) needs fp32 operands, and
// on the fp32 matrix cores 64 queries put it where HBM and matrix peak meet, so that form never gets
// close to the memory roofline.  Here every fp32 operand is written as the exact sum of three bf16
// numbers, x = x1 + x2 + x3 (x1 = bf16(x), x2 = bf16(x - x1), x3 = x - x1 - x2: 3 x 8 significant bits,
// each remainder exact in fp32), and the product e q is formed from the six piece products
// e1 q3, e1 q2, e2 q2, e1 q1, e2 q1, e3 q1 -- each exact in the fp32 accumulator -- on
// v_mfma_f32_32x32x16_bf16, which runs at 16 times the rate of the fp32 instruction: 6/16 of the matrix
// time, and the call becomes a stream over k and k_hat (or the codes) bound by HBM.
//
// Rounding: |x2| <= 2^-8 |x| and |x3| <= 2^-16 |x|, so the three piece products left out
// (e2 q3, e3 q2, e3 q3) are below (2^-24 + 2^-24 + 2^-32) |e q| per channel.  A run of 64 channels is
// 24 matrix instructions chained through one fp32 accumulator, each adding 16 exact products; the runs
// are added, the absolute value taken and the mean formed in fp64.  With every instruction off by at
// most two units in the last place of the run's sum of magnitudes a score stays within
// (2 + 2 * 24) * 2^-24 * sum_d |q_d e_d| of the exact one, inside the 65 * 2^-24 that the fp32
// matrix-core form guarantees, which is the bound stated for the call.
// Preconditions beyond finite inputs: as for the fp32 form, and |q|, |e| >= 2^-110 or 0 for the third
// pieces to stay normal bf16 numbers (smaller values lose their low bits).
//
// The queries are split once per call by split_queries_kernel into a workspace laid out in operand
// order -- [16-channel block][tile of 32 queries][piece][lane][8 bf16] -- so that a wavefront's B
// operand is one contiguous KiB straight from L2 into registers: no LDS, no vector-ALU work.  The keys
// go through LDS because the operand wants 32 tokens side by side while memory wants 512 contiguous
// bytes of one token: per chunk of 128 channels 256 lanes read k and k_hat [32 TT x 128] with 16-byte
// loads, subtract, split, and write three bf16 planes [32 TT][128 + 8] (row pitch 272 bytes: the 16-byte
// operand reads of 16 consecutive rows fall into different banks).  The planes are double-buffered, so
// one barrier per chunk is enough.  A workgroup owns 32 TT tokens x 32 NQ queries and has two kinds of
// wavefronts, four that stream and stage the keys and four that contract (see attn_split_kernel); a
// contracting wavefront takes query tile w % NQ over its 1/(4/NQ) of the chunk's channels for all TT
// token tiles, so it carries 16 TT fp32 sums and as many fp64 totals, and reloads a B operand's
// registers right after the last matrix instruction that reads them.
// Measured on [16384 x 8192] with 64 queries: 0.19 ms for the call against 0.21-0.28 ms on the fp32 matrix
// cores and 0.134 ms for the bytes at 8 TB/s; [131072 x 8192]: 1.33 against 1.65 ms (6.45 TB/s).
#include <atomic>
#include <type_traits>
#include <utility>

#include "kvq_internal.h"
#include "kvq_reduce.h"

namespace kvq {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr int kTok = 32;            // tokens of one 32x32 matrix tile (a workgroup owns TT of them)
constexpr int kCh = 128;            // channels staged per step
constexpr int kPitchH = kCh + 8;    // LDS row pitch in bf16 elements (272 bytes)
constexpr int kPlane = kTok * kPitchH;  // one piece of one buffer, in bf16 elements
constexpr int kRowsPerPass = kBlock / (kCh / 4);  // 8 rows of 32 sixteen-byte pieces per fill pass
constexpr int kPasses = kTok / kRowsPerPass;       // 4
constexpr uint32_t kOperandBytes = 64 * 16;        // one matrix operand: 64 lanes x 8 bf16

template <int... I, typename F>
__device__ __forceinline__ void unroll_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void unroll(F&& f) {
  unroll_impl(std::make_integer_sequence<int, N>{}, f);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(const void* base, int64_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// two fp32 numbers -> their nearest bf16 numbers packed in one word (a in the low half), and the
// exact remainders
__device__ __forceinline__ uint32_t peel(float& a, float& b) {
  const f32x2 v = {a, b};
  const bf16x2 p = __builtin_convertvector(v, bf16x2);
  uint32_t w;
  __builtin_memcpy(&w, &p, 4);
  a -= __uint_as_float(w << 16);
  b -= __uint_as_float(w & 0xffff0000u);
  return w;
}

// Queries in operand order: out[((kb * qtiles + n) * 3 + piece) * 64 + lane] holds the 8 bf16 pieces of
// query 32 n + lane % 32, channels 16 kb + 8 (lane / 32) .. + 7; rows past Q are zeros.
__global__ __launch_bounds__(kBlock) void split_queries_kernel(const float* __restrict__ queries, int64_t Q, int64_t D,
                                                               uint32_t qtiles, uint32_t operands,
                                                               u32x4* __restrict__ out) {
  const uint32_t idx = blockIdx.x * kBlock + threadIdx.x;
  const uint32_t lane = idx & 63, op = idx >> 6;
  if (op >= operands) return;
  const uint32_t n = op % qtiles, kb = op / qtiles;
  const int64_t query = (int64_t)n * 32 + (lane & 31);
  const int64_t d0 = (int64_t)kb * 16 + 8 * (lane >> 5);
  float v[8];
#pragma unroll
  for (int i = 0; i < 8; i++) v[i] = 0.0f;
  if (query < Q) {
    const f32x4 lo = *reinterpret_cast<const f32x4*>(queries + query * D + d0);
    const f32x4 hi = *reinterpret_cast<const f32x4*>(queries + query * D + d0 + 4);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      v[i] = lo[i];
      v[4 + i] = hi[i];
    }
  }
  u32x4* const dst = out + (size_t)op * 3 * 64 + lane;
#pragma unroll
  for (int piece = 0; piece < 3; piece++) {
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; i++) w[i] = peel(v[2 * i], v[2 * i + 1]);
    dst[piece * 64] = w;
  }
}

constexpr int kSets = 2;  // chunks of k and k_hat a streaming wavefront keeps in flight (even: set i % 2 goes to LDS buffer i % 2)

// LDS of attn_split_kernel<NQ, TT, .>: two buffers of three bf16 planes of 32 TT tokens, the partial scores
// that the wavefronts with a later share of the channels hand over ([PAR][CP - 1][NQ][TT][16][64] doubles; two
// alternating copies when a tile may be a single chunk long), eight doubles for the final sum
constexpr size_t split_planes_bytes(int TT) { return sizeof(uint16_t) * 2 * 3 * TT * kPlane; }
constexpr size_t split_comb_doubles(int NQ, int TT) { return (size_t)(4 / NQ - 1) * NQ * TT * 16 * 64; }
constexpr size_t split_lds_bytes(int NQ, int TT) {
  return split_planes_bytes(TT) + sizeof(double) * ((TT == 1 ? 2 : 1) * split_comb_doubles(NQ, TT) + 8);
}

// One workgroup per compute unit, eight wavefronts in two roles that meet at one barrier per chunk:
// wavefronts 4-7 stream k and k_hat (loads kSets chunks ahead, subtract, split, write the bf16 planes of the
// chunk after the one being contracted), wavefronts 0-3 contract the staged chunk with the query pieces, which
// they load themselves one chunk ahead.  A wavefront that did both would find its query operands (a
// microsecond away in L2) queued behind key loads, because loads return to a wavefront in the order it issued
// them; apart, neither role waits for the other's memory.  The workgroup walks its tiles (blockIdx.x,
// + gridDim.x, ...) as one sequence of chunks, so the stream runs ahead across tile boundaries too.
// A tile is 32 TT tokens x 32 NQ queries.  TT = 2 halves the query bytes per key byte (a query operand in
// registers feeds both token tiles): every byte goes through L2, which delivers about 13 TB/s on this part,
// and with one token tile the six bytes per query element and 32 tokens alone are 1.5 times the key stream.
template <int NQ, int TT, bool FROM_CODES>
__global__ __launch_bounds__(2 * kBlock, 1) void attn_split_kernel(const void* __restrict__ qsplit, uint32_t qtiles,
                                                                   const float* __restrict__ k,
                                                                   const float* __restrict__ k_hat,
                                                                   const int8_t* __restrict__ codes,
                                                                   const float* __restrict__ scales, int64_t N,
                                                                   int64_t D, uint32_t qchunks, uint32_t tiles,
                                                                   double* __restrict__ sums) {
  constexpr int CP = 4 / NQ;            // wavefronts that share a query tile split the channels CP ways
  constexpr int KB = (kCh / 16) / CP;   // 16-channel blocks per wavefront and chunk
  constexpr int RUN = 64 / (KB * 16);   // chunks per fp32 accumulation run of 64 channels
  constexpr int P = kPasses * TT;       // fill passes of 8 rows per chunk
  constexpr int PAR = TT == 1 ? 2 : 1;  // copies of the hand-over area (the host gives TT = 2 tiles of two chunks and more)
  constexpr int kTilePlane = TT * kPlane;
  constexpr size_t kComb = split_comb_doubles(NQ, TT);
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* const planes = reinterpret_cast<uint16_t*>(smem);                       // [2][3][32 TT][kPitchH]
  double* const comb = reinterpret_cast<double*>(smem + split_planes_bytes(TT));    // [PAR][CP - 1][NQ][TT][16][64]
  double* const red = comb + PAR * kComb;                                           // [8]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const uint32_t nchunks = (uint32_t)(D / kCh);
  const uint32_t my_tiles = (tiles - blockIdx.x + gridDim.x - 1) / gridDim.x;  // >= 1: the grid has at most `tiles` workgroups
  // chunks in this workgroup's sequence, and the groups of kSets chunks that cover them
  const uint64_t steps = (uint64_t)my_tiles * nchunks, groups = (steps + kSets - 1) / kSets;
  auto next_chunk = [&](uint32_t c) { return c + 1 == nchunks ? 0u : c + 1; };
  // Workgroups start their sweep over the channels at different chunks, so that they do not all ask for
  // the same lines of the queries at the same moment (the order of the chunks does not matter to the sum).
  auto first_chunk = [&](uint32_t tile) { return (uint32_t)((uint64_t)(tile / qchunks) * 5u % nchunks); };
  double total = 0.0;

  if (wave >= 4) {
    // ------------------------------------------------------------------ streaming wavefronts
    const int st = tid - kBlock;
    const int frow = st >> 5, fcol = (st & 31) * 4;
    uint32_t voff[P];  // byte offset of this lane's piece of each pass from the tile's first row
#pragma unroll
    for (int p = 0; p < P; p++) voff[p] = (uint32_t)(((int64_t)(frow + p * kRowsPerPass) * D + fcol) * 4);
    u32x4 kv[kSets][P], hv[kSets][P], sv[kSets];
    uint32_t wv[kSets][P];

    // where the next loads go: tile, chunks of it done, chunk; rows past the end of the matrix come back as
    // zeros from the descriptors' range check
    uint32_t ld_tile = blockIdx.x, ld_left = my_tiles, ld_done = 0, ld_chunk = 0;
    __amdgpu_buffer_rsrc_t kr, hr, sr;
    if constexpr (FROM_CODES) sr = buffer_of(scales, D * 4);
    auto open_tile = [&]() {
      const int64_t t0 = (int64_t)(ld_tile / qchunks) * (kTok * TT);
      const int64_t rows = N - t0 > kTok * TT ? kTok * TT : N - t0;
      kr = buffer_of(k + t0 * D, rows * D * 4);
      if constexpr (FROM_CODES) hr = buffer_of(codes + t0 * D, rows * D);
      else hr = buffer_of(k_hat + t0 * D, rows * D * 4);
      ld_chunk = first_chunk(ld_tile);
    };
    open_tile();
    auto issue = [&](auto set_tag) {
      constexpr int S = decltype(set_tag)::value;
      const uint32_t soff = ld_chunk * (kCh * 4);
#pragma unroll
      for (int p = 0; p < P; p++) kv[S][p] = __builtin_amdgcn_raw_buffer_load_b128(kr, (int)voff[p], (int)soff, 2);
      if constexpr (FROM_CODES) {
#pragma unroll
        for (int p = 0; p < P; p++)
          wv[S][p] = __builtin_amdgcn_raw_buffer_load_b32(hr, (int)(voff[p] >> 2), (int)(soff >> 2), 2);
        sv[S] = __builtin_amdgcn_raw_buffer_load_b128(sr, fcol * 4, (int)soff, 0);
      } else {
#pragma unroll
        for (int p = 0; p < P; p++) hv[S][p] = __builtin_amdgcn_raw_buffer_load_b128(hr, (int)voff[p], (int)soff, 2);
      }
      // (past the last chunk of the last tile the loads go on over that tile, unused: with every load
      // unconditional the compiler can count how many are in flight and waits for one set at a time)
      if (++ld_done == nchunks) {
        ld_done = 0;
        if (ld_left > 1) {
          ld_left--;
          ld_tile += gridDim.x;
          open_tile();
        } else {
          ld_chunk = first_chunk(ld_tile);
        }
      } else {
        ld_chunk = next_chunk(ld_chunk);
      }
    };
    // e = k - k_hat of the chunk in register set S, as three bf16 planes of LDS buffer S % 2
    auto stage = [&](auto set_tag) {
      constexpr int S = decltype(set_tag)::value;
      uint16_t* const base = planes + (S & 1) * 3 * kTilePlane + frow * kPitchH + fcol;
#pragma unroll
      for (int p = 0; p < P; p++) {
        float e[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
          float kh;
          if constexpr (FROM_CODES) kh = (float)((int)(wv[S][p] << (24 - 8 * i)) >> 24) * __uint_as_float(sv[S][i]);
          else kh = __uint_as_float(hv[S][p][i]);
          e[i] = __uint_as_float(kv[S][p][i]) - kh;
        }
#pragma unroll
        for (int piece = 0; piece < 3; piece++) {
          u32x2 w;
          w.x = peel(e[0], e[1]);
          w.y = peel(e[2], e[3]);
          *reinterpret_cast<u32x2*>(base + piece * kTilePlane + p * kRowsPerPass * kPitchH) = w;
        }
      }
    };
    unroll<kSets>([&](auto s) { issue(s); });
    // chunk i of the sequence sits in register set i % kSets and goes to LDS buffer i % 2; barrier i + 1
    // follows its staging.  The sequence is rounded up to whole groups of kSets chunks (the extra ones
    // restage the last tile, unread; the contracting wavefronts just meet the barriers), so the loop has no
    // exits between the sets and the compiler's count of loads in flight stays exact.
    for (uint64_t g = 0; g < groups; g++) {
      unroll<kSets>([&](auto s) {
        stage(s);
        issue(s);
        __syncthreads();
      });
    }
    __syncthreads();  // the contracting wavefronts' last partial scores are in LDS
  } else {
    // ---------------------------------------------------------------- contracting wavefronts
    const int nw = wave % NQ, cpart = wave / NQ;
    const int r = lane & 31, h = lane >> 5;
    const uint32_t qblock = qtiles * 3 * kOperandBytes;  // bytes of the query pieces of one 16-channel block
    const __amdgpu_buffer_rsrc_t qd = buffer_of(qsplit, (int64_t)(D / 16) * qblock);
    // this wavefront's B operands of a chunk: block b, piece j at  qoff + (8 chunk + b) qblock + j KiB
    auto qoff_of = [&](uint32_t tile) {
      return (uint32_t)lane * 16 + (uint32_t)(cpart * KB) * qblock + ((tile % qchunks) * NQ + (uint32_t)nw) * 3 * kOperandBytes;
    };
    u32x4 qop[KB][3];
    auto fetch_q = [&](uint32_t qoff, uint32_t chunk_soff, auto b_tag, auto j_tag) {
      constexpr int B = decltype(b_tag)::value, J = decltype(j_tag)::value;
      qop[B][J] = __builtin_amdgcn_raw_buffer_load_b128(qd, (int)(qoff + J * kOperandBytes),
                                                        (int)(chunk_soff + (uint32_t)B * qblock), 0);
    };
    uint32_t tile = blockIdx.x, chunk = first_chunk(tile), qoff = qoff_of(tile);
    unroll<KB>([&](auto b) { unroll<3>([&](auto j) { fetch_q(qoff, chunk * 8 * qblock, b, j); }); });
    f32x16 acc[TT];
    double acc64[TT][16];
#pragma unroll
    for (int t = 0; t < TT; t++)
#pragma unroll
      for (int i = 0; i < 16; i++) acc64[t][i] = 0.0;
    // A finished tile's partial scores stay in acc64 until the barrier that follows; the wavefronts with a
    // later share of the channels have put theirs into LDS before it, and after it the wavefronts with the
    // first share add everything up in a fixed order.  (The hand-over area is written again at the end of
    // the next tile: two barriers later, or into the other copy where a tile may be a single chunk.)
    bool pending = false;
    uint32_t par = 0, buf = 0;
    auto combine = [&]() {
      if (cpart == 0) {
        const double* const c = comb + (size_t)(par ^ (PAR - 1)) * kComb;
#pragma unroll
        for (int t = 0; t < TT; t++)
#pragma unroll
          for (int i = 0; i < 16; i++) {
            double s = acc64[t][i];
#pragma unroll
            for (int w = 0; w < CP - 1; w++) s += c[(((w * NQ + nw) * TT + t) * 16 + i) * 64 + lane];
            total += fabs(s);
          }
      }
#pragma unroll
      for (int t = 0; t < TT; t++)
#pragma unroll
        for (int i = 0; i < 16; i++) acc64[t][i] = 0.0;
      pending = false;
    };
    for (uint32_t left = my_tiles; left; left--, tile += gridDim.x) {
      int in_run = 0;
      for (uint32_t cc = 0; cc < nchunks; cc++) {
        // the operands to fetch meanwhile: the next chunk's, of this tile or the next (after the very last
        // chunk this one's once more, unused: cheaper than a branch around every load)
        uint32_t nchunk = chunk, nqoff = qoff;
        if (cc + 1 < nchunks) {
          nchunk = next_chunk(chunk);
        } else if (left > 1) {
          nchunk = first_chunk(tile + gridDim.x);
          nqoff = qoff_of(tile + gridDim.x);
        }
        const uint32_t soff = nchunk * 8 * qblock;
        __syncthreads();  // this chunk's planes are in LDS buffer `buf`
        if (pending) combine();
        const uint16_t* const ap = planes + buf * 3 * kTilePlane + r * kPitchH + cpart * KB * 16 + 8 * h;
        unroll<KB>([&](auto b_tag) {
          constexpr int B = decltype(b_tag)::value;
          bf16x8 a[TT][3];
#pragma unroll
          for (int t = 0; t < TT; t++)
#pragma unroll
            for (int j = 0; j < 3; j++) {
              const u32x4 w = *reinterpret_cast<const u32x4*>(ap + j * kTilePlane + t * kPlane + 16 * B);
              __builtin_memcpy(&a[t][j], &w, 16);
            }
          auto step = [&](int ai, auto j_tag, bool first) {
            constexpr int J = decltype(j_tag)::value;
            bf16x8 b;
            __builtin_memcpy(&b, &qop[B][J], 16);
#pragma unroll
            for (int t = 0; t < TT; t++) {
              if (first) {
                // a run starts from zero: the constant operand saves clearing 16 registers
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t][ai], b, zero, 0, 0, 0);
              } else {
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t][ai], b, acc[t], 0, 0, 0);
              }
            }
          };
          using J0 = std::integral_constant<int, 0>;
          using J1 = std::integral_constant<int, 1>;
          using J2 = std::integral_constant<int, 2>;
          // smallest products first; after the last use of a query piece its registers take the next chunk's
          step(0, J2{}, B == 0 && in_run == 0);
          __builtin_amdgcn_sched_barrier(0);
          fetch_q(nqoff, soff, b_tag, J2{});
          __builtin_amdgcn_sched_barrier(0);
          step(0, J1{}, false);
          step(1, J1{}, false);
          __builtin_amdgcn_sched_barrier(0);
          fetch_q(nqoff, soff, b_tag, J1{});
          __builtin_amdgcn_sched_barrier(0);
          step(0, J0{}, false);
          step(1, J0{}, false);
          step(2, J0{}, false);
          __builtin_amdgcn_sched_barrier(0);
          fetch_q(nqoff, soff, b_tag, J0{});
          __builtin_amdgcn_sched_barrier(0);
        });
        if (++in_run == RUN || cc + 1 == nchunks) {
          // the run's fp32 sums join the fp64 totals
#pragma unroll
          for (int t = 0; t < TT; t++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc64[t][i] += (double)acc[t][i];
          in_run = 0;
        }
        chunk = nchunk;
        qoff = nqoff;
        buf ^= 1;
      }
      // the wavefronts of a query tile hold the partial scores of their share of the channels
      if (cpart > 0) {
        double* const c = comb + (size_t)par * kComb;
#pragma unroll
        for (int t = 0; t < TT; t++)
#pragma unroll
          for (int i = 0; i < 16; i++) c[((((cpart - 1) * NQ + nw) * TT + t) * 16 + i) * 64 + lane] = acc64[t][i];
      }
      pending = true;
      par ^= PAR - 1;
    }
    for (uint64_t extra = groups * kSets - steps; extra; extra--) __syncthreads();  // the stream's padding
    __syncthreads();
    combine();
  }
  total = wave_sum(total);
  if (lane == 0) red[wave] = total;
  __syncthreads();
  if (tid == 0) sums[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

}  // namespace

// The score-error kernels need more dynamic LDS than a kernel gets by default: raise the limit of every
// instantiation, once per device (also from kvq_prepare_stream, so that nothing but launches is left for a
// stream capture).
kvq_status prepare_attn_split() {
  static std::atomic<uint64_t> done{0};
  int dev = -1;
  KVQ_HIP(hipGetDevice(&dev));
  const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t)1 << dev : 0;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return KVQ_OK;
#define KVQ_RAISE_LDS(NQ_, TT_, FC_)                                                                        \
  static_assert(split_lds_bytes(NQ_, TT_) <= 160 * 1024, "LDS of one compute unit");                       \
  KVQ_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_split_kernel<NQ_, TT_, FC_>),             \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)split_lds_bytes(NQ_, TT_)))
  KVQ_RAISE_LDS(2, 2, true);
  KVQ_RAISE_LDS(2, 2, false);
  KVQ_RAISE_LDS(2, 1, true);
  KVQ_RAISE_LDS(2, 1, false);
  KVQ_RAISE_LDS(1, 1, true);
  KVQ_RAISE_LDS(1, 1, false);
#undef KVQ_RAISE_LDS
  if (bit) done.fetch_or(bit, std::memory_order_release);
  return KVQ_OK;
}

bool attn_split_applicable(int64_t Q, int64_t D) {
  if (D % kCh != 0 || D > ((int64_t)1 << 22)) return false;  // the 64 rows of a tile within a 31-bit byte count
  const int64_t NQ = Q > 32 ? 2 : 1;
  const int64_t qtiles = (Q + 32 * NQ - 1) / (32 * NQ) * NQ;  // whole query chunks, padded with zero rows
  return qtiles * 32 * D * 6 <= kColmaxFloats * 4;
}

// queries, k, k_hat (or codes, scales) as for launch_attn_score_error; the caller has checked
// attn_split_applicable and 16-byte (codes: 4-byte) alignment of every pointer
kvq_status launch_attn_split(const float* queries, int64_t Q, const float* k, const float* k_hat,
                             const int8_t* codes, const float* scales, int64_t N, int64_t D, const Workspace& ws,
                             int* blocks_out, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  if (kvq_status s = prepare_attn_split()) return s;
  const int NQ = Q > 32 ? 2 : 1;
  // 64-token tiles where there are two query tiles to feed, a tile is two chunks or longer (the kernel's
  // single hand-over area relies on it) and every compute unit still gets a tile
  const int TT = (NQ == 2 && D >= 2 * kCh && (N + 2 * kTok - 1) / (2 * kTok) >= dev.cus) ? 2 : 1;
  const int64_t qchunks = (Q + 32 * NQ - 1) / (32 * NQ);
  const int64_t qtiles = qchunks * NQ;
  const int64_t ttiles = (N + kTok * TT - 1) / (kTok * TT);
  if (qchunks > INT32_MAX / 2 || ttiles > INT32_MAX / qchunks) return KVQ_ERR_OVERFLOW;
  const int64_t tiles = qchunks * ttiles;
  int64_t blocks = dev.cus < kMaxPartials ? dev.cus : kMaxPartials;  // one workgroup per compute unit
  if (blocks > tiles) blocks = tiles;
  const int64_t operands = (D / 16) * qtiles;  // x 3 pieces x 1 KiB <= 16 MiB
  hipLaunchKernelGGL(split_queries_kernel, dim3((uint32_t)((operands * 64 + kBlock - 1) / kBlock)), dim3(kBlock), 0,
                     stream, queries, Q, D, (uint32_t)qtiles, (uint32_t)operands,
                     reinterpret_cast<u32x4*>(ws.colmax));
  KVQ_HIP(hipGetLastError());
  const dim3 grid((uint32_t)blocks), block(2 * kBlock);
  const bool from_codes = k_hat == nullptr;
#define KVQ_LAUNCH_SPLIT(NQ_, TT_, FC_)                                                                          \
  do {                                                                                                           \
    constexpr size_t lds = split_lds_bytes(NQ_, TT_);                                                            \
    hipLaunchKernelGGL((attn_split_kernel<NQ_, TT_, FC_>), grid, block, lds, stream, (const void*)ws.colmax,     \
                       (uint32_t)qtiles, k, k_hat, codes, scales, N, D, (uint32_t)qchunks, (uint32_t)tiles,      \
                       ws.sums);                                                                                 \
  } while (0)
  if (NQ == 2 && TT == 2) {
    if (from_codes) KVQ_LAUNCH_SPLIT(2, 2, true);
    else KVQ_LAUNCH_SPLIT(2, 2, false);
  } else if (NQ == 2) {
    if (from_codes) KVQ_LAUNCH_SPLIT(2, 1, true);
    else KVQ_LAUNCH_SPLIT(2, 1, false);
  } else {
    if (from_codes) KVQ_LAUNCH_SPLIT(1, 1, true);
    else KVQ_LAUNCH_SPLIT(1, 1, false);
  }
#undef KVQ_LAUNCH_SPLIT
  KVQ_HIP(hipGetLastError());
  *blocks_out = (int)blocks;
  return KVQ_OK;
}

}  // namespace kvq
