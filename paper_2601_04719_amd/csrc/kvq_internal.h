// Internal declarations shared by the translation units of libkvq.so.
// Not part of the public ABI (that is include/kvq.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvq.h"
#include "kvq_bench.h"

namespace kvq {

constexpr int kBlock = 256;     // threads per workgroup of the reduction kernels: 4 wavefronts of 64
constexpr int kMaxBlock = 512;  // largest workgroup the codec kernels may be launched with

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// How a [batch, N, D] problem is cut into workgroups.
//
// A workgroup is TX x TY lanes (TX * TY = block threads, both powers of two).  Lane
// (tx, ty) owns the V consecutive channels starting at (ctile*TX + tx) * V and
// walks down the rows r0 + ty, r0 + ty + TY, ... of its row chunk, so whatever
// is per-channel (scales, running maxima) stays in registers for the whole
// walk, and a wavefront always touches whole contiguous row segments.
struct Tiling {
  int V;                   // channels per lane (1 = generic scalar path)
  int block;               // threads per workgroup
  int tx_log2;             // TX = 1 << tx_log2
  int64_t groups;          // ceil(D / V): lane-columns per row
  uint32_t ctiles;         // ceil(groups / TX)
  uint32_t rchunks;        // row chunks per slab
  int64_t rows_per_chunk;  // multiple of TY * unroll (last chunk may be short)
  int64_t items;           // batch * rchunks * ctiles = work items
};

// unroll: rows each lane keeps in flight.  passes > 0: every workgroup makes that
// many passes of TY * unroll rows; passes == 0: the row chunking is chosen to give
// about target_blocks work items.
Tiling make_tiling(int64_t batch, int64_t N, int64_t D, int V, int unroll, int64_t target_blocks,
                   int block = kBlock, int passes = 0);

// Launch shape of a streaming codec kernel (quantize / dequantize of any code format): lanes of V
// channels, `default_unroll` rows in flight per lane and `default_block` threads unless the options
// say otherwise, one-shot workgroups.  vector_lanes = false is the scalar fallback (one row at a time).
kvq_status stream_tiling(int64_t batch, int64_t N, int64_t D, int V, bool vector_lanes, int default_unroll,
                         int default_block, int* U_out, Tiling* t_out, int default_passes = 1);
// the same for a given number of compute units (host arithmetic only, no device needed)
kvq_status stream_tiling_for(int cus, int64_t batch, int64_t N, int64_t D, int V, bool vector_lanes,
                             int default_unroll, int default_block, int* U_out, Tiling* t_out,
                             int default_passes = 1);
// Launch shape of the fp32 scale reduction: J column groups per lane, U rows in flight, tiling in units of
// J * V channels per lane, row chunks limited to what the workspace holds.  vec = 16-byte row access.
// colmax_floats = size of the buffer that takes the per-row-chunk maxima.
kvq_status absmax_plan(int cus, int64_t batch, int64_t N, int64_t D, bool vec, int* J_out, int* U_out, Tiling* t_out,
                       int64_t colmax_floats = (int64_t)1 << 22);

// default launch shapes of the fp32 codec kernels: rows in flight per lane, threads per workgroup
constexpr int kQuantUnroll = 4, kQuantBlock = 512, kDequantUnroll = 2, kDequantBlock = 256;
// Rows narrower than a 256-lane workgroup (D < 1024) stack several rows per pass, so a workgroup writes one
// contiguous piece whatever its size; 512 lanes then do better for dequantize (16 KiB written per workgroup:
// [256 x 4096 x 128] 0.823 against 0.801 of peak in a sweep of workgroup size x rows in flight), while rows of
// 1024 channels and more prefer 256 ([16384 x 8192] 0.828 against 0.798).
inline int dequant_block_for(int64_t D) { return D < 1024 ? 512 : kDequantBlock; }

struct Options {
  int codec_width = 4;
  int codec_unroll = 0;  // 0 = per kernel default (quantize 4, dequantize 2)
  int blocks_per_cu = 0;  // 0 = per kernel default (error reductions: 1 dense, 2 from codes; codecs: 8)
  int nontemporal = 1;
  int block_threads = 0;  // 0 = per kernel default (quantize 512, dequantize 256)
  int passes_per_block = 1;
  int absmax_unroll = 8;
  int absmax_blocks_per_cu = 1;
  int absmax_span = 8;    // column groups per lane (1, 2, 4, 8), capped by the row width
  int absmax_passes = 0;  // 0 = long row chunks sized from blocks_per_cu
  int append_blocks_per_cu = 32;  // row chunking of the requantization pass of kvq_append
  int fused_min_lanes = 8;        // narrowest column tile of the single-pass fused kernel, in 16-byte lanes along a row
  int fused_max_rows = 0;         // rows a lane of that kernel holds: 4, 8, 16, or 0 = 8 where the tiles stay wide enough, else 16
  int fused_tall = 1;             // the persistent single-pass kernel that also keeps rows in LDS: 1 = where it is the faster form, 0 = never, 2 = as 1 but workgroups do not wait for their neighbours, 3 = wherever its tiles are more than half full
  int attn_form = 0;              // score-error contraction: 0 = bf16 pieces where the shape allows, 1 = fp32 matrix cores always
};
Options& options();

struct DeviceInfo {
  int device = -1;
  int cus = 0;
};
// Properties of the current device (cached); cus == 0 on failure.
DeviceInfo current_device();

// Records a failed HIP call for kvq_last_hip_error(); returns KVQ_ERR_HIP.
kvq_status hip_failed(hipError_t e);
#define KVQ_HIP(call)                                   \
  do {                                                  \
    hipError_t kvq_e_ = (call);                         \
    if (kvq_e_ != hipSuccess) return hip_failed(kvq_e_); \
  } while (0)

// batch, N, D >= 1 and batch * N * D elements indexable: KVQ_OK, KVQ_ERR_SHAPE or KVQ_ERR_OVERFLOW
kvq_status check_shape(int64_t batch, int64_t N, int64_t D);

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Largest lane width V in {16, 8, 4} (capped by `want`) such that rows of D fp32
// values / D int8 codes can be accessed with V-wide vectors, else 1.
int pick_width(int64_t D, const void* fp32_ptr, const void* int8_ptr, int want);

// Per-(device, stream) scratch: partial results of the error kernels, and the per-row-chunk column
// maxima of the scale reductions.
constexpr int kMaxPartials = 8192;
constexpr int64_t kColmaxFloats = (int64_t)1 << 22;  // 16 MiB
constexpr int kTickets = 1024;
struct Workspace {
  double* sums;   // [kMaxPartials]
  float* maxes;   // [kMaxPartials]
  float* colmax;  // [kColmaxFloats]: [row chunk][batch * D]
  uint32_t* tickets;  // [kTickets]: zero between launches (each kernel that counts in them leaves them at zero)
};
kvq_status get_workspace(hipStream_t stream, Workspace* out);
// frees the current device's workspace of `stream`, if there is one
kvq_status release_workspace(hipStream_t stream);

// ---- launchers (each validates nothing: the C-ABI layer has done that) ----
// scales = column absmax / qmax (127 for 8-bit codes, 7 for 4-bit codes)
// colmax = where the per-row-chunk maxima go, [row chunk][batch * D] within colmax_floats floats;
// nullptr = the stream's workspace (allocated on first use)
kvq_status launch_absmax_scales(const float* x, float* scales, int64_t batch, int64_t N, int64_t D,
                                hipStream_t stream, float qmax = 127.0f, float* colmax = nullptr,
                                int64_t colmax_floats = 0);
// second stage of a scale reduction that was split over row chunks:
// scales[i] = max_r colmax[r * total + i] / qmax
kvq_status launch_absmax_finalize(const float* colmax, float* scales, int64_t total, uint32_t rchunks, float qmax,
                                  hipStream_t stream);
// Row chunks a scale reduction over `total` = batch * D channels may use: bounded by the workspace.
inline int64_t absmax_chunk_cap(int64_t total) { return total > 0 ? kColmaxFloats / total : 0; }
// merges row chunks until at most `cap` (>= 1) remain
void limit_row_chunks(Tiling* t, int64_t batch, int64_t N, int64_t cap);
// 4-bit codes, two per byte (packed rows of D / 2 bytes); D is even.
kvq_status launch_quantize_int4(const float* x, const float* scales, uint8_t* packed, int64_t batch, int64_t N,
                                int64_t D, hipStream_t stream);
// slab b of x starts f_slab elements after slab b-1, of packed p_slab bytes (multiples of D and D / 2)
kvq_status launch_quantize_int4_strided(const float* x, const float* scales, uint8_t* packed, int64_t batch,
                                        int64_t N, int64_t D, int64_t f_slab, int64_t p_slab, hipStream_t stream);
kvq_status launch_dequantize_int4(const uint8_t* packed, const float* scales, float* x_hat, int64_t batch,
                                  int64_t N, int64_t D, hipStream_t stream);
// FP8 (OCP E4M3) codes, one byte per element; scales = absmax / 448.
kvq_status launch_quantize_fp8(const float* x, const float* scales, uint8_t* codes, int64_t batch, int64_t N,
                               int64_t D, hipStream_t stream);
kvq_status launch_dequantize_fp8(const uint8_t* codes, const float* scales, float* x_hat, int64_t batch, int64_t N,
                                 int64_t D, hipStream_t stream);
kvq_status launch_quantize(const float* x, const float* scales, int8_t* codes, int64_t batch, int64_t N,
                           int64_t D, hipStream_t stream);
// The same with separate slab pitches (in elements, multiples of D) for x and codes.
kvq_status launch_quantize_strided(const float* x, const float* scales, int8_t* codes, int64_t batch, int64_t N,
                                   int64_t D, int64_t x_slab, int64_t c_slab, hipStream_t stream);
// Streaming append: merge the new tokens' absmax into the scales, re-express cached codes of grown
// channels, quantize the new tokens behind them.
// scales_prev holds the new tokens' candidate scales on entry, the old scales on exit; scales = the larger
kvq_status launch_append_merge(float* scales, float* scales_prev, int64_t n, hipStream_t stream);
// 4-bit cache (packed rows of D / 2 bytes, D even), fp32 new tokens
kvq_status launch_append_int4(const float* x_new, float* scales, float* scales_prev, uint8_t* packed, int64_t batch,
                              int64_t n_old, int64_t m, int64_t capacity, int64_t D, hipStream_t stream);
kvq_status launch_append(const float* x_new, float* scales, float* scales_prev, int8_t* codes, int64_t batch,
                         int64_t n_old, int64_t m, int64_t capacity, int64_t D, hipStream_t stream);
// the same with fp16 / bf16 new tokens (dtype: KVQ_DTYPE_F16 or KVQ_DTYPE_BF16)
kvq_status launch_append_16(int dtype, const void* x_new, float* scales, float* scales_prev, int8_t* codes,
                            int64_t batch, int64_t n_old, int64_t m, int64_t capacity, int64_t D,
                            hipStream_t stream);
kvq_status launch_dequantize(const int8_t* codes, const float* scales, float* x_hat, int64_t batch,
                             int64_t N, int64_t D, hipStream_t stream);
// One-pass absmax + quantize for slabs that fit one workgroup's registers.
bool fused_slab_applicable(const float* x, const float* scales, const int8_t* codes, int64_t N, int64_t D);
bool fused_tall_applicable(const float* x, const float* scales, const int8_t* codes, int64_t batch, int64_t N,
                           int64_t D, bool slab_form);
kvq_status prepare_fused_tall();
kvq_status launch_fused_tall(const float* x, float* scales, int8_t* codes, int64_t batch, int64_t N, int64_t D,
                             const Workspace& ws, hipStream_t stream);
kvq_status launch_fused_slab(const float* x, float* scales, int8_t* codes, int64_t batch, int64_t N, int64_t D,
                             hipStream_t stream);
kvq_status launch_quantize_variant(int variant, const float* x, const float* scales, int8_t* codes,
                                   int64_t batch, int64_t N, int64_t D, hipStream_t stream);
kvq_status launch_probe_codec(int mode, const float* src_f32, float* dst_f32, const int8_t* src_i8,
                              int8_t* dst_i8, const float* scales, int64_t batch, int64_t N, int64_t D,
                              hipStream_t stream);
kvq_status launch_scores_from_codes(const float* queries, int64_t Q, const int8_t* codes, const float* scales,
                                    int64_t batch, int64_t N, int64_t D, float* out, hipStream_t stream);
// Matrix-core form of the same for Q >= 3 (16-byte aligned codes; D % 64 == 0 up to 1024, D % 256 == 0 up to 8192).
bool scores_mfma_applicable(const float* queries, int64_t Q, const int8_t* codes, const float* scales, int64_t D);
kvq_status launch_scores_mfma(const float* queries, int64_t Q, const int8_t* codes, const float* scales,
                              int64_t batch, int64_t N, int64_t D, float* out, hipStream_t stream);
// Scores from a 4-bit cache (packed rows of D / 2 bytes, D even).
kvq_status launch_scores_from_codes_int4(const float* queries, int64_t Q, const uint8_t* packed, const float* scales,
                                         int64_t batch, int64_t N, int64_t D, float* out, hipStream_t stream);
kvq_status launch_absmax_scales_16(int dtype, const void* x, float* scales, int64_t batch, int64_t N, int64_t D,
                                   hipStream_t stream);
kvq_status launch_quantize_16(int dtype, const void* x, const float* scales, int8_t* codes, int64_t batch,
                              int64_t N, int64_t D, hipStream_t stream);
// slab b of x starts x_slab elements after slab b-1, of codes c_slab (both multiples of D)
kvq_status launch_quantize_16_strided(int dtype, const void* x, const float* scales, int8_t* codes, int64_t batch,
                                      int64_t N, int64_t D, int64_t x_slab, int64_t c_slab, hipStream_t stream);
kvq_status launch_dequantize_16(int dtype, const int8_t* codes, const float* scales, void* x_hat, int64_t batch,
                                int64_t N, int64_t D, hipStream_t stream);
kvq_status launch_roundtrip_error_dense(const float* x, const float* x_hat, int64_t count, double* sumsq_out,
                                        float* maxabs_out, hipStream_t stream);
kvq_status launch_roundtrip_error_codes(const float* x, const int8_t* codes, const float* scales,
                                        int64_t batch, int64_t N, int64_t D, double* sumsq_out,
                                        float* maxabs_out, hipStream_t stream);
// folds n per-workgroup partials in index order: *sum_out = sum / divisor, *max_out = max (maxes, max_out may be null)
kvq_status launch_fold_partials(const double* sums, const float* maxes, int n, double divisor, double* sum_out,
                                float* max_out, hipStream_t stream);
kvq_status launch_attn_score_error(const float* queries, int64_t Q, const float* k, const float* k_hat,
                                   const int8_t* codes, const float* scales, int64_t N, int64_t D,
                                   double* mean_abs_out, hipStream_t stream);
// The same contraction on the bf16 matrix cores (every fp32 operand as the exact sum of three bf16 pieces): D a
// multiple of 128, every pointer 16-byte (codes: 4-byte) aligned, and the split queries (6 bytes per element of
// whole 32- or 64-query chunks) within the workspace's 16 MiB.  Leaves *blocks_out partial sums in ws.sums.
bool attn_split_applicable(int64_t Q, int64_t D);
// one-time set-up of those kernels on the current device (their LDS limit); called by the launcher as well
kvq_status prepare_attn_split();
kvq_status launch_attn_split(const float* queries, int64_t Q, const float* k, const float* k_hat,
                             const int8_t* codes, const float* scales, int64_t N, int64_t D, const Workspace& ws,
                             int* blocks_out, hipStream_t stream);

// ---- device helpers ----
#ifdef __HIPCC__
// 16-bit input formats: tags, and exact / round-to-nearest-even conversions on raw bit patterns
struct f16_tag {};
struct bf16_tag {};

typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));

// ---- element conversions -----------------------------------------------------------------
template <typename T>
__device__ __forceinline__ float widen(uint16_t bits);
template <>
__device__ __forceinline__ float widen<f16_tag>(uint16_t bits) {
  _Float16 h;
  __builtin_memcpy(&h, &bits, 2);
  return (float)h;
}
template <>
__device__ __forceinline__ float widen<bf16_tag>(uint16_t bits) {
  return __uint_as_float((uint32_t)bits << 16);
}

// round to nearest even (finite inputs)
template <typename T>
__device__ __forceinline__ uint16_t narrow(float v);
template <>
__device__ __forceinline__ uint16_t narrow<f16_tag>(float v) {
  const _Float16 h = (_Float16)v;
  uint16_t bits;
  __builtin_memcpy(&bits, &h, 2);
  return bits;
}
template <>
__device__ __forceinline__ uint16_t narrow<bf16_tag>(float v) {
  const uint32_t u = __float_as_uint(v);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(T* p, T v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
}

// Rounding without a convert instruction: once a value is clamped to a range inside [-2^22, 2^22],
// adding 1.5 * 2^23 rounds it to the nearest integer with ties to even (the sum lies in [2^23, 2^24)
// where the spacing is 1, and 1.5 * 2^23 is even) and leaves the two's-complement integer in the low
// bits of the sum's bit pattern.
constexpr float kRoundMagic = 12582912.0f;

// Divisor for a channel: its scale, or +inf for a zero scale (x / inf = +-0 -> code 0).
__device__ __forceinline__ float divisor_of(float s) { return s == 0.0f ? __builtin_inff() : s; }

// The fp32 quotient x / div without the divide.  r approximates 1 / div to within 2^-50 relative (fp64), so
// (double)x * r is within 2^-26 fp32-ulps of x / div.  A quotient of two fp32 numbers is never
// closer than 2^-25 ulp to a midpoint between two adjacent fp32 numbers (write x = A 2^a, div = B 2^b
// with 24-bit integers A, B and a midpoint as M 2^m with M odd: x/div - M 2^m = (A 2^a - B M 2^(b+m)) /
// (B 2^b) has a nonzero integer multiple of a power of two on top and B < 2^24 below; it cannot be 0
// because B M has an odd factor beyond 24 bits), in the subnormal and overflow ranges as well, so
// rounding the product to fp32 gives exactly the correctly rounded fp32 quotient: the same bits as
// x / div, with 3 instructions per element instead of the 11-12 of the IEEE divide sequence.  Used
// where a kernel is bound by the vector ALUs rather than by HBM.
__device__ __forceinline__ float quotient_by(float x, double r) { return (float)((double)x * r); }

// 1 / div in fp64 to within a few 2^-53: hardware estimate, three Newton steps (each squares the
// relative error, so even a 7-bit estimate would do; one rounding per fma).  div = +-inf (the divisor of a zero scale) gives 0, as x / inf.
__device__ __forceinline__ double reciprocal_of(float div) {
  const double d = (double)div;
  double r = __builtin_amdgcn_rcp(d);
  r = fma(fma(-d, r, 1.0), r, r);
  r = fma(fma(-d, r, 1.0), r, r);
  r = fma(fma(-d, r, 1.0), r, r);
  return __builtin_isinf(div) ? 0.0 : r;
}


// Decomposition of a work-item index into (slab, row chunk, column tile).
struct Item {
  int64_t slab;
  int64_t row0, row1;   // rows [row0, row1) of the slab
  int64_t group;        // lane-column index of this lane (may be >= groups: inactive)
  int ty, TY;
};
__device__ __forceinline__ Item decode_item(uint32_t item, uint32_t ctiles, uint32_t rchunks,
                                            int64_t rows_per_chunk, int64_t N, int tx_log2) {
  Item it;
  const uint32_t ct = item % ctiles;
  const uint32_t rest = item / ctiles;
  const uint32_t rc = rest % rchunks;
  it.slab = rest / rchunks;
  const int tid = threadIdx.x;
  const int tx = tid & ((1 << tx_log2) - 1);
  it.ty = tid >> tx_log2;
  it.TY = (int)blockDim.x >> tx_log2;
  it.group = (int64_t)ct * (1 << tx_log2) + tx;
  it.row0 = (int64_t)rc * rows_per_chunk;
  it.row1 = it.row0 + rows_per_chunk;
  if (it.row1 > N) it.row1 = N;
  return it;
}
#endif

}  // namespace kvq
