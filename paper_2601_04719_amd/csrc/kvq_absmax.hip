// Scale computation: scales[b,d] = max_t |x[b,t,d]| / 127
// (paper: Eq. (scale), Eq. (scale_compute), Algorithm "Compute Scales").
//
// The paper computes scales on the host only.  Here the column maximum is a
// streaming reduction over rows: every lane owns V adjacent channels, reads
// its rows with 16-byte loads that a wavefront issues as whole contiguous row
// segments, keeps V running maxima in registers, and at the end the maxima of
// the lanes that share channels are combined in LDS.  A workgroup that saw
// every row of its slab divides and writes the scales itself; otherwise it
// stores its maxima to its row chunk's slot of a workspace with plain vector
// stores and a small second kernel takes the maximum over the chunks and
// divides.  (Merging with one atomic max per channel and workgroup instead
// costs about 80 ns per workgroup once the channels fall into a few cache
// lines -- 20 us of a 26 us call on [32768 x 128] -- and needs the scale
// buffer cleared first.)  max is associative and commutative, so the result
// does not depend on the launch shape.
//
// Unlike the codec kernels, workgroups here walk long row chunks: one workgroup
// per compute unit, each lane owning up to 8 column groups so that the workgroup
// reads whole rows -- one fat contiguous stream per compute unit.  Measured on
// the 1B-element shape: 7.0 TB/s, against 6.5 TB/s with eight 4 KiB-wide
// workgroups per compute unit, and 4 TB/s for one-shot workgroups of a few rows
// (measured when every workgroup still ended in an atomic per channel).
#include <mutex>
#include <type_traits>

#include "kvq_internal.h"

namespace kvq {

// Second stage: scales[i] = max over row chunks of colmax[r * total + i], then one IEEE fp32 divide
// by qmax (127 for 8-bit codes, 7 for 4-bit codes, 448 for FP8).  A workgroup owns kFinX adjacent
// channels; its kFinY lanes per channel split the row chunks and meet in LDS.
constexpr int kFinX = 16, kFinY = kBlock / kFinX;
__global__ __launch_bounds__(kBlock) void absmax_finalize_kernel(const float* __restrict__ colmax,
                                                                 float* __restrict__ scales, int64_t total,
                                                                 uint32_t rchunks, float qmax) {
  __shared__ float red[kBlock];
  const int tx = threadIdx.x % kFinX, ty = threadIdx.x / kFinX;
  const int64_t i = (int64_t)blockIdx.x * kFinX + tx;
  float m = 0.0f;
  if (i < total) {
    const float* p = colmax + i;
    uint32_t r = ty;
    for (; r + 3 * kFinY < rchunks; r += 4 * kFinY) {
      const float a = p[(int64_t)r * total], b = p[(int64_t)(r + kFinY) * total];
      const float c = p[(int64_t)(r + 2 * kFinY) * total], d = p[(int64_t)(r + 3 * kFinY) * total];
      m = fmaxf(fmaxf(m, fmaxf(a, b)), fmaxf(c, d));
    }
    for (; r < rchunks; r += kFinY) m = fmaxf(m, p[(int64_t)r * total]);
  }
  red[threadIdx.x] = m;
  __syncthreads();
  if (ty == 0 && i < total) {
    for (int y = 1; y < kFinY; y++) m = fmaxf(m, red[y * kFinX + tx]);
    scales[i] = m / qmax;
  }
}

// |v| joins the running maximum only when strictly larger, as in the algorithm;
// fmaxf(m, |v|) is the same function on finite data.
__device__ __forceinline__ float absmax_step(float m, float v) { return fmaxf(m, fabsf(v)); }

// A lane owns J groups of V adjacent channels, TX groups apart: with J * TX * V
// >= D a workgroup reads whole rows, i.e. one contiguous stream per workgroup.
template <int V, int J, int U, bool NT>
__global__ __launch_bounds__(kBlock) void absmax_kernel(const float* __restrict__ x, float* __restrict__ dst,
                                                        int64_t chunk_stride, float qmax, int64_t N, int64_t D,
                                                        int tx_log2, uint32_t ctiles, uint32_t rchunks,
                                                        int64_t rows_per_chunk, int64_t groups) {
  __shared__ float red[J == 1 ? kBlock * V : 1];
  // decode_item numbers column tiles in units of TX groups; a tile here is J of those
  Item it = decode_item(blockIdx.x, ctiles, rchunks, rows_per_chunk, N, tx_log2);
  const int TX = 1 << tx_log2;
  const int64_t group0 = (it.group - (threadIdx.x & (TX - 1))) * J + (threadIdx.x & (TX - 1));
  float m[J][V];
#pragma unroll
  for (int j = 0; j < J; j++)
#pragma unroll
    for (int i = 0; i < V; i++) m[j][i] = 0.0f;
  bool act[J];
#pragma unroll
  for (int j = 0; j < J; j++) act[j] = group0 + (int64_t)j * TX < groups;

  if (act[0]) {
    const float* base = x + (it.slab * N) * D + group0 * V;
    const int64_t step = (int64_t)it.TY * D;  // elements between successive rows of this lane
    int64_t row = it.row0 + it.ty;
    const float* p = base + row * D;
    if constexpr (V == 4) {
      auto do_rows = [&](auto tag) {
        constexpr int R = decltype(tag)::value;
        f32x4 v[R][J];
#pragma unroll
        for (int u = 0; u < R; u++)
#pragma unroll
          for (int j = 0; j < J; j++)
            if (J == 1 || act[j]) v[u][j] = ld<NT>(reinterpret_cast<const f32x4*>(p + u * step) + (int64_t)j * TX);
            else v[u][j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < R; u++)
#pragma unroll
          for (int j = 0; j < J; j++) {
            m[j][0] = absmax_step(m[j][0], v[u][j].x);
            m[j][1] = absmax_step(m[j][1], v[u][j].y);
            m[j][2] = absmax_step(m[j][2], v[u][j].z);
            m[j][3] = absmax_step(m[j][3], v[u][j].w);
          }
      };
      for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, p += U * step)
        do_rows(std::integral_constant<int, U>{});
      for (; row < it.row1; row += it.TY, p += step) do_rows(std::integral_constant<int, 1>{});
    } else {
      static_assert(V == 1 && J == 1, "absmax lanes are 4-wide or scalar");
      for (; row + (int64_t)(U - 1) * it.TY < it.row1; row += (int64_t)U * it.TY, p += U * step) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; u++) v[u] = p[u * step];
#pragma unroll
        for (int u = 0; u < U; u++) m[0][0] = absmax_step(m[0][0], v[u]);
      }
      for (; row < it.row1; row += it.TY, p += step) m[0][0] = absmax_step(m[0][0], *p);
    }
  }

  // combine the TY lanes that share a channel group (LDS; only rows narrower than a workgroup
  // have TY > 1, and those use J == 1)
  if constexpr (J == 1) {
    if (it.TY > 1) {
#pragma unroll
      for (int i = 0; i < V; i++) red[i * kBlock + threadIdx.x] = m[0][i];
      __syncthreads();
      if (it.ty == 0) {
        for (int y = 1; y < it.TY; y++) {
#pragma unroll
          for (int i = 0; i < V; i++) m[0][i] = fmaxf(m[0][i], red[i * kBlock + y * TX + threadIdx.x]);
        }
      }
    }
  }
  // rchunks == 1: dst is the scale buffer and this workgroup has the final maxima;
  // otherwise dst is the workspace, [row chunk][batch * D], and chunk_stride = batch * D
  if (it.ty == 0) {
    const bool final_pass = rchunks == 1;
    const uint32_t rc = (blockIdx.x / ctiles) % rchunks;
#pragma unroll
    for (int j = 0; j < J; j++) {
      if (!act[j]) continue;
      float* out = dst + (int64_t)rc * chunk_stride + it.slab * D + (group0 + (int64_t)j * TX) * V;
      if (final_pass) {
#pragma unroll
        for (int i = 0; i < V; i++) out[i] = m[j][i] / qmax;
      } else if constexpr (V == 4) {
        *reinterpret_cast<f32x4*>(out) = f32x4{m[j][0], m[j][1], m[j][2], m[j][3]};
      } else {
#pragma unroll
        for (int i = 0; i < V; i++) out[i] = m[j][i];
      }
    }
  }
}

template <int V, int J, int U>
static kvq_status launch_absmax_t(const float* x, float* dst, int64_t chunk_stride, float qmax, int64_t N,
                                  int64_t D, const Tiling& t, bool nt, hipStream_t stream) {
  const dim3 grid((uint32_t)t.items), block(kBlock);
  if (nt)
    hipLaunchKernelGGL((absmax_kernel<V, J, U, true>), grid, block, 0, stream, x, dst, chunk_stride, qmax, N, D,
                       t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
  else
    hipLaunchKernelGGL((absmax_kernel<V, J, U, false>), grid, block, 0, stream, x, dst, chunk_stride, qmax, N, D,
                       t.tx_log2, t.ctiles, t.rchunks, t.rows_per_chunk, t.groups);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

kvq_status absmax_plan(int cus, int64_t batch, int64_t N, int64_t D, bool vec, int* J_out, int* U_out, Tiling* t_out,
                       int64_t colmax_floats) {
  const Options& o = options();
  const int V = vec ? 4 : 1;
  // J column groups per lane: as many as it takes for a workgroup to span whole rows, at most 8.
  // Measured on D = 8192 (J = 1 / 4 / 8, one workgroup per compute unit): 4096 rows 37 / 30 / 35 us,
  // 16384 rows 85.6 / 84.6 / 86.4 us, 65536 rows 337 / 312 / 313 us, 131072 rows 700 / 663 / 610 us:
  // 4 up to about 2^30 elements, 8 from there.
  int J = 1;
  if (V == 4) {
    const int64_t groups = D / 4;
    const int64_t elements = batch * N * D;
    const int jmax = elements >= ((int64_t)cus << 22) ? 8 : 4;
    while (J < o.absmax_span && J < jmax && (int64_t)kBlock * J < groups) J *= 2;
  }
  // rows in flight: with several column groups per lane J * U 16-byte loads, at most 8 (16 measured 1-4 % slower on D = 8192 with
  // 16384 to 131072 rows, 32 slower still: one workgroup per compute unit wants a short loop, not depth)
  int U = o.absmax_unroll;
  if (J >= 2)
    while (J * U > 8 && U > 1) U /= 2;
  int passes = o.absmax_passes;
  // tiling in units of J * V channels per lane
  Tiling t = make_tiling(batch, N, D, V * J, U, (int64_t)cus * o.absmax_blocks_per_cu, kBlock, passes);
  while (t.items > ((int64_t)1 << 30) && passes > 0 && passes < (1 << 20)) {
    passes *= 2;
    t = make_tiling(batch, N, D, V * J, U, (int64_t)cus * o.absmax_blocks_per_cu, kBlock, passes);
  }
  if (J > 1) {
    // make_tiling sized TX for D / (V*J) lane-columns; with J > 1 rows are at least a workgroup wide
    t.tx_log2 = 8;
    t.groups = D / V;
    t.ctiles = (uint32_t)((t.groups + (int64_t)kBlock * J - 1) / ((int64_t)kBlock * J));
    t.items = batch * (int64_t)t.rchunks * t.ctiles;
  }
  limit_row_chunks(&t, batch, N, colmax_floats / (batch * D));
  if (t.items > INT32_MAX) return KVQ_ERR_OVERFLOW;
  *J_out = J;
  *U_out = U;
  *t_out = t;
  return KVQ_OK;
}

kvq_status launch_absmax_scales(const float* x, float* scales, int64_t batch, int64_t N, int64_t D,
                                hipStream_t stream, float qmax, float* colmax, int64_t colmax_floats) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  const Options& o = options();
  const int V = (D % 4 == 0 && aligned(x, 16)) ? 4 : 1;
  int J, U;
  Tiling t;
  if (colmax == nullptr) colmax_floats = kColmaxFloats;
  if (kvq_status s = absmax_plan(dev.cus, batch, N, D, V == 4, &J, &U, &t, colmax_floats)) return s;
  const int64_t total = batch * D;
  float* dst = scales;
  if (t.rchunks > 1) {
    if (colmax == nullptr) {
      Workspace ws;
      if (kvq_status s = get_workspace(stream, &ws)) return s;
      colmax = ws.colmax;
    }
    dst = colmax;
  }
  const bool nt = o.nontemporal != 0;
  kvq_status s;
#define KVQ_AM(V_, J_, U_) s = launch_absmax_t<V_, J_, U_>(x, dst, total, qmax, N, D, t, nt, stream)
  if (V == 4 && J == 8) KVQ_AM(4, 8, 1);
  else if (V == 4 && J == 4) KVQ_AM(4, 4, 2);
  else if (V == 4 && J == 2) KVQ_AM(4, 2, 4);
  else if (V == 4 && U == 4) KVQ_AM(4, 1, 4);
  else if (V == 4 && U == 8) KVQ_AM(4, 1, 8);
  else if (V == 4) KVQ_AM(4, 1, 16);
  else if (U == 4) KVQ_AM(1, 1, 4);
  else if (U == 8) KVQ_AM(1, 1, 8);
  else KVQ_AM(1, 1, 16);
#undef KVQ_AM
  if (s != KVQ_OK) return s;
  if (t.rchunks > 1) return launch_absmax_finalize(dst, scales, total, t.rchunks, qmax, stream);
  return KVQ_OK;
}

kvq_status launch_absmax_finalize(const float* colmax, float* scales, int64_t total, uint32_t rchunks, float qmax,
                                  hipStream_t stream) {
  const int64_t blocks = (total + kFinX - 1) / kFinX;
  if (blocks > INT32_MAX) return KVQ_ERR_OVERFLOW;
  hipLaunchKernelGGL(absmax_finalize_kernel, dim3((uint32_t)blocks), dim3(kBlock), 0, stream, colmax, scales, total,
                     rchunks, qmax);
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

// ------------------------------------------------------------ the scale reduction without an allocation
// For callers that cannot allocate (code under HIP graph capture, serving loops, harnesses that forbid
// it): the per-row-chunk maxima go to a fixed array in device memory instead of the per-stream workspace.
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process
// ends.  In host code the array's name only stands for the symbol; the address kernels can use is asked
// from the runtime once per device and kept.
static __device__ __align__(256) float scratch[KVQ_STATIC_SCRATCH_FLOATS];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices];  // per device: device address of `scratch`, null until asked

kvq_status static_scratch(float** out) {
  int dev = -1;
  KVQ_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return hip_failed(hipErrorInvalidDevice);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    KVQ_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return hip_failed(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return KVQ_OK;
}
}  // namespace

void limit_row_chunks(Tiling* t, int64_t batch, int64_t N, int64_t cap) {
  if (cap < 1) cap = 1;
  if ((int64_t)t->rchunks <= cap) return;
  // keep rows_per_chunk a multiple of what it already is a multiple of: scale it by a whole factor
  const int64_t factor = ((int64_t)t->rchunks + cap - 1) / cap;
  t->rows_per_chunk *= factor;
  t->rchunks = (uint32_t)((N + t->rows_per_chunk - 1) / t->rows_per_chunk);
  t->items = batch * (int64_t)t->rchunks * t->ctiles;
}

}  // namespace kvq

// The entry point lives in this file, next to the array, the look-up of its address and the kernels
// that take that address as an argument.
extern "C" kvq_status kvq_absmax_scales_static(const float* x, float* scales, int64_t batch, int64_t N, int64_t D,
                                               kvq_stream_t stream) {
  using namespace kvq;
  if (!x || !scales) return KVQ_ERR_NULL;
  if (kvq_status s = check_shape(batch, N, D)) return s;
  // every (slab, channel) needs one slot per row chunk
  if (batch * D > (int64_t)KVQ_STATIC_SCRATCH_FLOATS) return KVQ_ERR_LIMIT;
  float* ptr = nullptr;
  if (kvq_status s = static_scratch(&ptr)) return s;
  // Nothing in the array has to start at zero: every workgroup of the first stage stores the maxima of
  // all channels of its (row chunk, slab, column tile), and the second stage reads exactly those slots.
  return launch_absmax_scales(x, scales, batch, N, D, stream, 127.0f, ptr, (int64_t)KVQ_STATIC_SCRATCH_FLOATS);
}
