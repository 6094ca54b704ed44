// C-ABI layer of libkvq.so: argument validation, launch-shape choice, the
// per-stream workspace.  No arithmetic of the method lives here.
#include <limits.h>

#include <map>
#include <mutex>
#include <utility>

#include "kvq_internal.h"

namespace kvq {

static thread_local int g_last_hip_error = 0;

kvq_status hip_failed(hipError_t e) {
  g_last_hip_error = (int)e;
  (void)hipGetLastError();  // clear the sticky launch error so later calls start clean
  return KVQ_ERR_HIP;
}

Options& options() {
  // per host thread: a thread sweeping launch options changes its own launches only, and no lock is needed
  static thread_local Options o;
  return o;
}

DeviceInfo current_device() {
  // a fixed table, so that a call never allocates host memory either
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static DeviceInfo cache[kMaxDevices];
  DeviceInfo info;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return info;
  std::lock_guard<std::mutex> lock(mu);
  if (cache[dev].cus > 0) return cache[dev];
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return info;
  info.device = dev;
  info.cus = cus;
  cache[dev] = info;
  return info;
}

int pick_width(int64_t D, const void* fp32_ptr, const void* int8_ptr, int want) {
  for (int V = 16; V >= 4; V >>= 1) {
    if (V > want) continue;
    if (D % V) continue;
    // a lane moves V fp32 values as 16-byte vectors and V codes as one V-byte vector
    if (fp32_ptr && !aligned(fp32_ptr, 16)) continue;
    if (int8_ptr && !aligned(int8_ptr, (uintptr_t)V)) continue;
    return V;
  }
  return 1;
}

static int ceil_log2(int64_t v) {
  int l = 0;
  while (((int64_t)1 << l) < v) l++;
  return l;
}

Tiling make_tiling(int64_t batch, int64_t N, int64_t D, int V, int unroll, int64_t target_blocks, int block,
                   int passes) {
  Tiling t;
  t.V = V;
  t.block = block;
  t.groups = (D + V - 1) / V;
  t.tx_log2 = t.groups >= block ? ceil_log2(block) : ceil_log2(t.groups);
  const int64_t TX = (int64_t)1 << t.tx_log2;
  const int64_t TY = block / TX;
  const int64_t ctiles = (t.groups + TX - 1) / TX;
  const int64_t step = TY * unroll;  // rows one pass of the workgroup covers
  const int64_t fixed = batch * ctiles;
  const int64_t max_chunks = (N + step - 1) / step;
  int64_t want_chunks = (target_blocks + fixed - 1) / fixed;
  if (passes > 0) want_chunks = (max_chunks + passes - 1) / passes;
  if (want_chunks > max_chunks) want_chunks = max_chunks;
  if (want_chunks < 1) want_chunks = 1;
  int64_t rows = (N + want_chunks - 1) / want_chunks;
  rows = (rows + step - 1) / step * step;
  t.rows_per_chunk = rows;
  const int64_t rchunks = (N + rows - 1) / rows;
  t.ctiles = (uint32_t)ctiles;
  t.rchunks = (uint32_t)rchunks;
  t.items = batch * rchunks * ctiles;
  return t;
}

kvq_status stream_tiling(int64_t batch, int64_t N, int64_t D, int V, bool vector_lanes, int default_unroll,
                         int default_block, int* U_out, Tiling* t_out, int default_passes) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  return stream_tiling_for(dev.cus, batch, N, D, V, vector_lanes, default_unroll, default_block, U_out, t_out,
                           default_passes);
}

kvq_status stream_tiling_for(int cus, int64_t batch, int64_t N, int64_t D, int V, bool vector_lanes,
                             int default_unroll, int default_block, int* U_out, Tiling* t_out, int default_passes) {
  const Options o = options();
  int U = o.codec_unroll > 0 ? o.codec_unroll : default_unroll;
  if (!vector_lanes) U = 1;
  else if (V > 4 && U > 4) U = 4;
  // the passes option, when moved off its default of 1, overrides a kernel's own default
  int passes = o.passes_per_block != 1 ? o.passes_per_block : default_passes;
  const int block = o.block_threads > 0 ? o.block_threads : default_block;
  const int64_t target = (int64_t)cus * (o.blocks_per_cu > 0 ? o.blocks_per_cu : 8);  // used when passes == 0
  Tiling t = make_tiling(batch, N, D, V, U, target, block, passes);
  // one-shot workgroups by default; fall back to longer walks only when the grid would not be indexable
  while (t.items > ((int64_t)1 << 30) && passes > 0 && passes < (1 << 20)) {
    passes *= 2;
    t = make_tiling(batch, N, D, V, U, target, block, passes);
  }
  if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
  *U_out = U;
  *t_out = t;
  return KVQ_OK;
}

namespace {
std::mutex g_ws_mutex;
std::map<std::pair<int, hipStream_t>, Workspace> g_ws_table;
}  // namespace

kvq_status get_workspace(hipStream_t stream, Workspace* out) {
  int dev = -1;
  KVQ_HIP(hipGetDevice(&dev));
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  auto key = std::make_pair(dev, stream);
  auto it = g_ws_table.find(key);
  if (it != g_ws_table.end()) {
    *out = it->second;
    return KVQ_OK;
  }
  void* p = nullptr;
  KVQ_HIP(hipMalloc(&p, (size_t)kMaxPartials * (sizeof(double) + sizeof(float)) + (size_t)kColmaxFloats * sizeof(float) +
                            (size_t)kTickets * sizeof(uint32_t)));
  Workspace w;
  w.sums = static_cast<double*>(p);
  w.maxes = reinterpret_cast<float*>(w.sums + kMaxPartials);
  w.colmax = w.maxes + kMaxPartials;
  w.tickets = reinterpret_cast<uint32_t*>(w.colmax + kColmaxFloats);
  if (hipError_t e = hipMemsetAsync(w.tickets, 0, (size_t)kTickets * sizeof(uint32_t), stream)) {
    (void)hipFree(p);
    return hip_failed(e);
  }
  g_ws_table[key] = w;
  *out = w;
  return KVQ_OK;
}

kvq_status release_workspace(hipStream_t stream) {
  int dev = -1;
  KVQ_HIP(hipGetDevice(&dev));
  void* p = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    auto it = g_ws_table.find(std::make_pair(dev, stream));
    if (it == g_ws_table.end()) return KVQ_OK;
    p = it->second.sums;  // start of the one allocation
    g_ws_table.erase(it);
  }
  KVQ_HIP(hipFree(p));
  return KVQ_OK;
}

// batch, N, D >= 1 and batch*N*D (in bytes of fp32) indexable in int64 / size_t.
kvq_status check_shape(int64_t batch, int64_t N, int64_t D) {
  if (batch < 1 || N < 1 || D < 1) return KVQ_ERR_SHAPE;
  const int64_t lim = INT64_MAX / 8;  // room for the 4-byte element size and headroom
  if (N > lim / D) return KVQ_ERR_OVERFLOW;
  if (batch > lim / (N * D)) return KVQ_ERR_OVERFLOW;
  if (batch > INT32_MAX / 2 || D > ((int64_t)1 << 40)) return KVQ_ERR_OVERFLOW;
  if (batch * D > lim) return KVQ_ERR_OVERFLOW;
  return KVQ_OK;
}

}  // namespace kvq

using namespace kvq;

extern "C" {

kvq_status kvq_absmax_scales(const float* x, float* scales, int64_t batch, int64_t N, int64_t D,
                             kvq_stream_t stream) {
  if (!x || !scales) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  return launch_absmax_scales(x, scales, batch, N, D, stream);
}

kvq_status kvq_quantize(const float* x, const float* scales, int8_t* codes, int64_t batch, int64_t N,
                        int64_t D, kvq_stream_t stream) {
  if (!x || !scales || !codes) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  return launch_quantize(x, scales, codes, batch, N, D, stream);
}

kvq_status kvq_dequantize(const int8_t* codes, const float* scales, float* x_hat, int64_t batch, int64_t N,
                          int64_t D, kvq_stream_t stream) {
  if (!codes || !scales || !x_hat) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  return launch_dequantize(codes, scales, x_hat, batch, N, D, stream);
}

kvq_status kvq_absmax_scales_t(int dtype, const void* x, float* scales, int64_t batch, int64_t N, int64_t D,
                               kvq_stream_t stream) {
  if (!x || !scales) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (dtype == KVQ_DTYPE_F32) return launch_absmax_scales(static_cast<const float*>(x), scales, batch, N, D, stream);
  if (dtype != KVQ_DTYPE_F16 && dtype != KVQ_DTYPE_BF16) return KVQ_ERR_ARG;
  if (!aligned(x, 2)) return KVQ_ERR_ARG;
  return launch_absmax_scales_16(dtype, x, scales, batch, N, D, stream);
}

kvq_status kvq_quantize_t(int dtype, const void* x, const float* scales, int8_t* codes, int64_t batch, int64_t N,
                          int64_t D, kvq_stream_t stream) {
  if (!x || !scales || !codes) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (dtype == KVQ_DTYPE_F32) return launch_quantize(static_cast<const float*>(x), scales, codes, batch, N, D, stream);
  if (dtype != KVQ_DTYPE_F16 && dtype != KVQ_DTYPE_BF16) return KVQ_ERR_ARG;
  if (!aligned(x, 2)) return KVQ_ERR_ARG;
  return launch_quantize_16(dtype, x, scales, codes, batch, N, D, stream);
}

kvq_status kvq_dequantize_t(int dtype, const int8_t* codes, const float* scales, void* x_hat, int64_t batch,
                            int64_t N, int64_t D, kvq_stream_t stream) {
  if (!codes || !scales || !x_hat) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (dtype == KVQ_DTYPE_F32) return launch_dequantize(codes, scales, static_cast<float*>(x_hat), batch, N, D, stream);
  if (dtype != KVQ_DTYPE_F16 && dtype != KVQ_DTYPE_BF16) return KVQ_ERR_ARG;
  if (!aligned(x_hat, 2)) return KVQ_ERR_ARG;
  return launch_dequantize_16(dtype, codes, scales, x_hat, batch, N, D, stream);
}

kvq_status kvq_absmax_scales_int4(const float* x, float* scales, int64_t batch, int64_t N, int64_t D,
                                  kvq_stream_t stream) {
  if (!x || !scales) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  return launch_absmax_scales(x, scales, batch, N, D, stream, 7.0f);
}

kvq_status kvq_quantize_int4(const float* x, const float* scales, uint8_t* packed, int64_t batch, int64_t N,
                             int64_t D, kvq_stream_t stream) {
  if (!x || !scales || !packed) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (D % 2) return KVQ_ERR_ARG;
  return launch_quantize_int4(x, scales, packed, batch, N, D, stream);
}

kvq_status kvq_dequantize_int4(const uint8_t* packed, const float* scales, float* x_hat, int64_t batch, int64_t N,
                               int64_t D, kvq_stream_t stream) {
  if (!packed || !scales || !x_hat) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (D % 2) return KVQ_ERR_ARG;
  return launch_dequantize_int4(packed, scales, x_hat, batch, N, D, stream);
}

kvq_status kvq_absmax_scales_fp8(const float* x, float* scales, int64_t batch, int64_t N, int64_t D,
                                 kvq_stream_t stream) {
  if (!x || !scales) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  return launch_absmax_scales(x, scales, batch, N, D, stream, 448.0f);
}

kvq_status kvq_quantize_fp8(const float* x, const float* scales, uint8_t* codes, int64_t batch, int64_t N,
                            int64_t D, kvq_stream_t stream) {
  if (!x || !scales || !codes) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  return launch_quantize_fp8(x, scales, codes, batch, N, D, stream);
}

kvq_status kvq_dequantize_fp8(const uint8_t* codes, const float* scales, float* x_hat, int64_t batch, int64_t N,
                              int64_t D, kvq_stream_t stream) {
  if (!codes || !scales || !x_hat) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  return launch_dequantize_fp8(codes, scales, x_hat, batch, N, D, stream);
}

kvq_status kvq_append(const float* x_new, float* scales, float* scales_prev, int8_t* codes, int64_t batch,
                      int64_t n_old, int64_t m, int64_t capacity, int64_t D, kvq_stream_t stream) {
  if (!x_new || !scales || !scales_prev || !codes) return KVQ_ERR_NULL;
  if (n_old < 0 || m < 1) return KVQ_ERR_SHAPE;
  if (kvq_status s = check_shape(batch, capacity, D)) return s;
  if (m > capacity || n_old > capacity - m) return KVQ_ERR_ARG;
  if (scales == scales_prev) return KVQ_ERR_ARG;
  return launch_append(x_new, scales, scales_prev, codes, batch, n_old, m, capacity, D, stream);
}

kvq_status kvq_prepare_stream(kvq_stream_t stream) {
  Workspace ws;
  if (kvq_status s = get_workspace(stream, &ws)) return s;
  if (kvq_status s = prepare_attn_split()) return s;
  return prepare_fused_tall();
}

kvq_status kvq_release_stream(kvq_stream_t stream) { return release_workspace(stream); }

kvq_status kvq_append_t(int dtype, const void* x_new, float* scales, float* scales_prev, int8_t* codes,
                        int64_t batch, int64_t n_old, int64_t m, int64_t capacity, int64_t D, kvq_stream_t stream) {
  if (dtype == KVQ_DTYPE_F32)
    return kvq_append(static_cast<const float*>(x_new), scales, scales_prev, codes, batch, n_old, m, capacity, D, stream);
  if (dtype != KVQ_DTYPE_F16 && dtype != KVQ_DTYPE_BF16) return KVQ_ERR_ARG;
  if (!x_new || !scales || !scales_prev || !codes) return KVQ_ERR_NULL;
  if (n_old < 0 || m < 1) return KVQ_ERR_SHAPE;
  if (kvq_status s = check_shape(batch, capacity, D)) return s;
  if (m > capacity || n_old > capacity - m) return KVQ_ERR_ARG;
  if (scales == scales_prev || !aligned(x_new, 2)) return KVQ_ERR_ARG;
  return launch_append_16(dtype, x_new, scales, scales_prev, codes, batch, n_old, m, capacity, D, stream);
}

kvq_status kvq_append_int4(const float* x_new, float* scales, float* scales_prev, uint8_t* packed, int64_t batch,
                           int64_t n_old, int64_t m, int64_t capacity, int64_t D, kvq_stream_t stream) {
  if (!x_new || !scales || !scales_prev || !packed) return KVQ_ERR_NULL;
  if (n_old < 0 || m < 1) return KVQ_ERR_SHAPE;
  if (kvq_status s = check_shape(batch, capacity, D)) return s;
  if (D % 2) return KVQ_ERR_ARG;
  if (m > capacity || n_old > capacity - m) return KVQ_ERR_ARG;
  if (scales == scales_prev) return KVQ_ERR_ARG;
  return launch_append_int4(x_new, scales, scales_prev, packed, batch, n_old, m, capacity, D, stream);
}

kvq_status kvq_quantize_fused(const float* x, float* scales, int8_t* codes, int64_t batch, int64_t N,
                              int64_t D, kvq_stream_t stream) {
  if (!x || !scales || !codes) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  // A slab whose column tiles fit one workgroup's registers (up to 2048 rows), or the registers and LDS of a
  // compute unit (up to 4096; also the faster form for many shorter slabs), is read once; anything taller
  // needs every row of a column before its first code can be written, i.e. two passes over x.  (Splitting the batch into groups small enough for the
  // 256 MiB memory-side cache was measured and gave no reuse.)
  const bool slab_form = fused_slab_applicable(x, scales, codes, N, D);
  if (fused_tall_applicable(x, scales, codes, batch, N, D, slab_form)) {
    Workspace ws;
    if (kvq_status s = get_workspace(stream, &ws)) return s;
    return launch_fused_tall(x, scales, codes, batch, N, D, ws, stream);
  }
  if (slab_form) return launch_fused_slab(x, scales, codes, batch, N, D, stream);
  if (kvq_status s = launch_absmax_scales(x, scales, batch, N, D, stream)) return s;
  return launch_quantize(x, scales, codes, batch, N, D, stream);
}

kvq_status kvq_roundtrip_error(const float* x, const float* x_hat, const int8_t* codes, const float* scales,
                               int64_t batch, int64_t N, int64_t D, double* sumsq_out, float* maxabs_out,
                               kvq_stream_t stream) {
  if (!x || !sumsq_out || !maxabs_out) return KVQ_ERR_NULL;
  if (!x_hat && (!codes || !scales)) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (!aligned(sumsq_out, 8) || !aligned(maxabs_out, 4)) return KVQ_ERR_ARG;
  if (x_hat) return launch_roundtrip_error_dense(x, x_hat, batch * N * D, sumsq_out, maxabs_out, stream);
  return launch_roundtrip_error_codes(x, codes, scales, batch, N, D, sumsq_out, maxabs_out, stream);
}

kvq_status kvq_attn_score_error(const float* queries, int64_t Q, const float* k, const float* k_hat,
                                const int8_t* codes, const float* scales, int64_t N, int64_t D,
                                double* mean_abs_out, kvq_stream_t stream) {
  if (!queries || !k || !mean_abs_out) return KVQ_ERR_NULL;
  if (!k_hat && (!codes || !scales)) return KVQ_ERR_NULL;
  if (Q < 1) return KVQ_ERR_SHAPE;
  if (kvq_status s = check_shape(1, N, D)) return s;
  if (Q > INT32_MAX || Q > (INT64_MAX / 8) / D) return KVQ_ERR_OVERFLOW;
  if (!aligned(mean_abs_out, 8)) return KVQ_ERR_ARG;
  return launch_attn_score_error(queries, Q, k, k_hat, codes, scales, N, D, mean_abs_out, stream);
}

kvq_status kvq_scores_from_codes(const float* queries, int64_t Q, const int8_t* codes, const float* scales,
                                 int64_t batch, int64_t N, int64_t D, float* scores_out, kvq_stream_t stream) {
  if (!queries || !codes || !scales || !scores_out) return KVQ_ERR_NULL;
  if (Q < 1) return KVQ_ERR_SHAPE;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (Q > INT32_MAX || Q > (INT64_MAX / 8) / D || batch > (INT64_MAX / 8) / (Q * D) || Q > (INT64_MAX / 8) / N ||
      batch > (INT64_MAX / 8) / (Q * N))
    return KVQ_ERR_OVERFLOW;
  return launch_scores_from_codes(queries, Q, codes, scales, batch, N, D, scores_out, stream);
}

kvq_status kvq_scores_from_codes_int4(const float* queries, int64_t Q, const uint8_t* packed, const float* scales,
                                      int64_t batch, int64_t N, int64_t D, float* scores_out, kvq_stream_t stream) {
  if (!queries || !packed || !scales || !scores_out) return KVQ_ERR_NULL;
  if (Q < 1) return KVQ_ERR_SHAPE;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  if (D % 2) return KVQ_ERR_ARG;
  if (Q > INT32_MAX || Q > (INT64_MAX / 8) / D || batch > (INT64_MAX / 8) / (Q * D) || Q > (INT64_MAX / 8) / N ||
      batch > (INT64_MAX / 8) / (Q * N))
    return KVQ_ERR_OVERFLOW;
  return launch_scores_from_codes_int4(queries, Q, packed, scales, batch, N, D, scores_out, stream);
}

const char* kvq_status_string(kvq_status status) {
  switch (status) {
    case KVQ_OK: return "KVQ_OK";
    case KVQ_ERR_NULL: return "KVQ_ERR_NULL: a required pointer is NULL";
    case KVQ_ERR_SHAPE: return "KVQ_ERR_SHAPE: batch, N, D and Q must be >= 1";
    case KVQ_ERR_OVERFLOW: return "KVQ_ERR_OVERFLOW: problem size is not indexable";
    case KVQ_ERR_HIP: return "KVQ_ERR_HIP: a HIP runtime call failed";
    case KVQ_ERR_ARG: return "KVQ_ERR_ARG: inconsistent or out-of-range argument";
    case KVQ_ERR_LIMIT: return "KVQ_ERR_LIMIT: problem exceeds the fixed scratch of an entry point that allocates nothing";
    default: return "unknown kvq status";
  }
}

int kvq_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
