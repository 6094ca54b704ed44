// Scale computation and quantization in one pass, with the column tile in the registers and LDS of a
// persistent workgroup (paper: Eq. (scale_compute) + Eq. (quant_op); same results as the two separate kernels).
//
// The single pass has to hold all N rows of the columns it works on.  Up to N = 2048 a column tile of
// 32 channels (one 128-byte line of x per row) fits the registers of a workgroup (kvq_fused.hip).  At
// N = 4096 such a tile is 512 KiB, the whole register file of a compute unit, so here one 512-lane
// workgroup owns the unit: each lane keeps 46 rows of 4 channels in registers (184 of its 256) and 18 more
// in a private slot of LDS (144 KiB in all).  With a single workgroup per unit nothing else hides the
// phases of a tile behind each other, so the workgroup is persistent and pipelines them itself: while it
// quantizes and stores the rows of one tile, register by register, it issues the loads of the next tile
// into the registers just freed.  Only the reduction of the column maxima (lane exchanges, one barrier)
// runs with nothing in flight.  The same 64 rows per lane make tiles of 64 channels x 2048 rows, 128 x 1024
// and 256 x 512; which problems take this kernel and which the register-only one is decided, from
// measurements, in fused_tall_applicable.
//
// All loads and stores go through buffer descriptors sized to the tile, so rows past N, channels past D
// and the tile after a workgroup's last one need no branches: loads beyond the descriptor return zero
// (which leaves a maximum of absolute values alone) and stores beyond it are dropped.
//
// A 32-channel tile's rows of codes are 32 bytes, a quarter of a cache line (64 channels: half); the other
// pieces are written by the workgroups that hold the neighbouring tiles.  Those run on the same XCD in the
// same turn and, before each tile, wait for each other for a bounded time (a hint for speed only), so that
// the pieces meet in L2.  Wider tiles write whole lines and stream them out.
#include <atomic>
#include <type_traits>
#include <utility>

#include "kvq_internal.h"

namespace kvq {

namespace {

constexpr int kTallBlock = 512;   // lanes: TX along a row (4 TX channels) x 512 / TX down the rows
constexpr int kTallRegRows = 46;  // rows per lane held in registers
constexpr int kTallLdsRows = 18;  // rows per lane held in LDS
constexpr int kTallBatches = 6;   // a tile's rows are worked through in this many batches
constexpr int kTallStage = (kTallLdsRows + kTallBatches - 1) / kTallBatches;  // rows staged on their way to LDS
constexpr int kTallRowsPerLane = kTallRegRows + kTallLdsRows;  // 64: a tile is up to 64 * 512 / TX rows tall
constexpr int kTallWaves = kTallBlock / 64;
constexpr size_t tall_lds_bytes(int tx) {
  return (size_t)kTallLdsRows * kTallBlock * 16 + 2 * (size_t)kTallWaves * tx * 16;
}
static_assert(tall_lds_bytes(64) <= 160 * 1024, "LDS of one compute unit");
constexpr int kTallXcds = 8;              // workgroup i of a launch is handed to XCD i % 8
constexpr int kTallPolls = 64;             // how often a workgroup looks for its neighbours before it goes on alone
constexpr uint32_t kOutside = 0x80000000u;  // an offset no descriptor reaches, whatever is added below 2^31

template <int... I, typename F>
__device__ __forceinline__ void tall_unroll_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void tall_unroll(F&& f) {
  tall_unroll_impl(std::make_integer_sequence<int, N>{}, f);
}

// A descriptor is the same for every lane; saying so keeps it in scalar registers across the loop.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tall_buffer(const void* base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  const uint64_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
  const uint64_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(lo | hi << 32), 0,
                                           __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000);
}

// Where a workgroup is in the sequence of tiles of its XCD.  Quads of adjacent column tiles (which share
// lines of codes) are dealt to the XCDs in turn, and the tiles of a quad are neighbours in an XCD's
// sequence, so they are in flight on compute units of the same XCD at the same time and their pieces of a
// line meet in its L2.  A workgroup keeps its place inside a quad and walks from quad to quad in steps the
// host has already divided into whole slabs and a rest, so the walk needs scalar additions only.
struct TallTile {
  uint32_t quad;         // number of the quad, slab-major; >= total_quads: no tile
  uint32_t slab;         // quad / quads_per_slab
  uint32_t quad_in_slab;  // quad % quads_per_slab
};

// TXLOG: log2 of the lanes along a row (8 to 64: tiles of 32 to 256 channels, up to 4096 down to 512 rows).
// NT: streaming stores, for tiles whose rows of codes are whole cache lines.
template <int TXLOG, bool NT>
__global__ __launch_bounds__(kTallBlock, 1) void fused_tall_kernel(const float* __restrict__ x,
                                                                   float* __restrict__ scales,
                                                                   int8_t* __restrict__ codes, uint32_t total_quads,
                                                                   uint32_t quads_per_slab, uint32_t quad_log2,
                                                                   uint32_t step_slabs, uint32_t step_quads,
                                                                   uint32_t N, uint32_t D,
                                                                   uint32_t* __restrict__ tickets) {
  constexpr int kTallTX = 1 << TXLOG, kTallTY = kTallBlock / kTallTX;
  static_assert(kTallTX >= 8 && kTallTX <= 64, "a wavefront holds every column group of the tile");
  extern __shared__ __align__(16) unsigned char tall_lds[];
  f32x4* const rows = reinterpret_cast<f32x4*>(tall_lds);       // [kTallLdsRows][kTallBlock], slot per lane
  f32x4* const red = rows + kTallLdsRows * kTallBlock;          // [2][kTallWaves][kTallTX]
  const uint32_t tid = threadIdx.x, tx = tid % kTallTX, ty = tid / kTallTX, wave = tid / 64, lane = tid % 64;
  const uint32_t xcd = blockIdx.x % kTallXcds, first = blockIdx.x / kTallXcds;
  const uint32_t column_tile = first & ((1u << quad_log2) - 1);  // this workgroup's place in every quad
  const uint32_t xstep = kTallTY * D * 4, cstep = kTallTY * D;  // bytes from a lane's row to its next one
  const int64_t slab_elems = (int64_t)N * D;

  f32x4 v[kTallRegRows];
  float m[4];
  double rcp[4];  // reciprocals of the held tile's divisors

  // Loads a tile (descriptor nx, this lane's first byte xo) while quantizing the tile held in v and LDS
  // into the codes behind cx at this lane's first byte co.  Leaves the column maxima of the loaded
  // rows in m.  In kTallBatches batches: a batch first quantizes its share of the rows held in LDS, which
  // frees their slots; moves the rows the batch before loaded for those slots from the staging registers
  // to LDS; loads its own rows for LDS into the staging registers; then quantizes its share of the rows
  // held in registers, loading the next tile's row into each register as it is freed.  Loads return in
  // order, so waiting for the staged rows of the batch before leaves everything younger in flight.
  auto turn = [&](__amdgpu_buffer_rsrc_t cx, uint32_t co, __amdgpu_buffer_rsrc_t nx, uint32_t xo) {
    auto encode = [&](const f32x4& r) {
      uint32_t w = 0;
#pragma unroll
      for (int i = 0; i < 4; i++) {
        float y = quotient_by(r[i], rcp[i]);  // the bits of r[i] / divisor, without the divide sequence
        y = __builtin_amdgcn_fmed3f(y, -127.0f, 127.0f);
        w |= (__float_as_uint(y + kRoundMagic) & 0xffu) << (8 * i);
      }
      return w;
    };
    auto fetch = [&](int row) {
      const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(nx, (int)(xo + (uint32_t)row * xstep), 0, 2);
      return __builtin_bit_cast(f32x4, w);
    };
    auto put = [&](const f32x4& r, int row) {
      __builtin_amdgcn_raw_buffer_store_b32(encode(r), cx, (int)(co + (uint32_t)row * cstep), 0, NT ? 2 : 0);
    };
    f32x4 staged[kTallStage];
#pragma unroll
    for (int i = 0; i < 4; i++) m[i] = 0.0f;
    auto hand_over = [&](auto B) {  // the staged rows of batch B: into the maxima and to their slots in LDS
      tall_unroll<kTallStage>([&](auto J) {
        constexpr int j = decltype(B)::value * kTallStage + decltype(J)::value;
        if constexpr (j < kTallLdsRows) {
#pragma unroll
          for (int i = 0; i < 4; i++) m[i] = fmaxf(m[i], fabsf(staged[decltype(J)::value][i]));
          rows[j * kTallBlock + tid] = staged[decltype(J)::value];
        }
      });
      // maxima may be taken in any order, and the compiler would rather take them all at the end and keep
      // the staged rows until then: have these here and now
      asm volatile("" : "+v"(m[0]), "+v"(m[1]), "+v"(m[2]), "+v"(m[3]));
    };
    tall_unroll<kTallBatches>([&](auto B) {
      constexpr int b = decltype(B)::value;
      tall_unroll<kTallStage>([&](auto J) {
        constexpr int j = b * kTallStage + decltype(J)::value;
        if constexpr (j < kTallLdsRows) put(rows[j * kTallBlock + tid], kTallRegRows + j);
      });
      // the fences keep the steps in this order: left alone, the compiler moves the hand-over to right
      // behind the staging loads and waits for them with little else in flight
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (b > 0) hand_over(std::integral_constant<int, (b > 0 ? b - 1 : 0)>{});
      __builtin_amdgcn_sched_barrier(0);
      tall_unroll<kTallStage>([&](auto J) {
        constexpr int j = b * kTallStage + decltype(J)::value;
        if constexpr (j < kTallLdsRows) staged[decltype(J)::value] = fetch(kTallRegRows + j);
      });
      __builtin_amdgcn_sched_barrier(0);
      constexpr int lo = b * kTallRegRows / kTallBatches, hi = (b + 1) * kTallRegRows / kTallBatches;
      tall_unroll<hi - lo>([&](auto U) {
        constexpr int u = lo + decltype(U)::value;
        put(v[u], u);
        v[u] = fetch(u);
      });
      __builtin_amdgcn_sched_barrier(0);
    });
    hand_over(std::integral_constant<int, kTallBatches - 1>{});
    __builtin_amdgcn_sched_barrier(0);
    tall_unroll<kTallRegRows>([&](auto U) {
      constexpr int u = decltype(U)::value;
#pragma unroll
      for (int i = 0; i < 4; i++) m[i] = fmaxf(m[i], fabsf(v[u][i]));
    });
  };

  // first channel and width (0: no such tile) of the workgroup's tile of a quad; descriptors of its x and codes
  auto first_channel_of = [&](const TallTile& t) {
    return ((t.quad_in_slab << quad_log2) + column_tile) * (kTallTX * 4);
  };
  auto width_of = [&](const TallTile& t) {
    const uint32_t c = first_channel_of(t);
    if (t.quad >= total_quads || c >= D) return 0u;
    return D - c < kTallTX * 4 ? D - c : (uint32_t)(kTallTX * 4);
  };
  auto x_of = [&](const TallTile& t) {
    const uint32_t w = width_of(t);
    return tall_buffer(x + t.slab * slab_elems + first_channel_of(t), w ? ((N - 1) * D + w) * 4 : 0);
  };
  auto codes_of = [&](const TallTile& t) {
    const uint32_t w = width_of(t);
    return tall_buffer(codes + t.slab * slab_elems + first_channel_of(t), w ? (N - 1) * D + w : 0);
  };

  // One turn more than the workgroup has tiles: the first quantizes nothing (an empty descriptor drops its
  // stores) and loads the first tile, the last loads nothing and quantizes the last tile.
  TallTile cur{total_quads, 0, 0};
  TallTile nxt;
  nxt.quad = xcd + kTallXcds * (first >> quad_log2);
  nxt.slab = (uint32_t)__builtin_amdgcn_readfirstlane((int)(nxt.quad / quads_per_slab));
  nxt.quad_in_slab = nxt.quad - nxt.slab * quads_per_slab;
#pragma unroll
  for (int u = 0; u < kTallRegRows; u++) v[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int i = 0; i < 4; i++) rcp[i] = 1.0;
  // The workgroups that hold the other tiles of the same quads (same XCD, same place in its sequence) write
  // the other pieces of the same lines of codes.  The pieces only meet in L2 if they are written within a
  // few microseconds of each other, and left alone the workgroups drift apart by more than that within a
  // few tiles (a line that leaves L2 in pieces costs several times its share of the write bandwidth).  So
  // before each tile's stores a workgroup takes a ticket from the quads' counter and waits, for a bounded
  // number of polls, until its neighbours have taken theirs.  Nothing depends on the wait but speed: when
  // the bound is reached the workgroup goes on.  After its last tile a workgroup takes one more ticket, and
  // whoever takes the very last one puts the counter back to zero for the next launch.
  uint32_t* const ticket = tickets ? tickets + (xcd * (gridDim.x / kTallXcds >> quad_log2) + (first >> quad_log2)) : nullptr;
  const uint32_t neighbours = 1u << quad_log2;
  uint32_t turns = 0;
  uint32_t parity = 0;
  for (;;) {
    const uint32_t cw = width_of(cur), nw = width_of(nxt);
    const uint32_t co = tx * 4 < cw ? ty * D + tx * 4 : kOutside;
    const uint32_t xo = tx * 4 < nw ? ty * D * 4 + tx * 16 : kOutside;
    turn(codes_of(cur), co, x_of(nxt), xo);
    if (nxt.quad >= total_quads) break;  // nothing was loaded: the tile just written was the last (same for all lanes)
    turns++;
    cur = nxt;
    nxt.quad += step_slabs * quads_per_slab + step_quads;
    nxt.slab += step_slabs;
    nxt.quad_in_slab += step_quads;
    if (nxt.quad_in_slab >= quads_per_slab) {
      nxt.quad_in_slab -= quads_per_slab;
      nxt.slab += 1;
    }

    // column maxima: over the lanes of a wavefront that share a column group, then over the wavefronts
#pragma unroll
    for (int i = 0; i < 4; i++) {
#pragma unroll
      for (int s = kTallTX; s < 64; s <<= 1) m[i] = fmaxf(m[i], __shfl_xor(m[i], s));
    }
    f32x4* const slot = red + parity * (kTallWaves * kTallTX);
    if (lane < kTallTX) slot[wave * kTallTX + lane] = f32x4{m[0], m[1], m[2], m[3]};
    __syncthreads();
    f32x4 top = slot[tx];
#pragma unroll
    for (int w = 1; w < kTallWaves; w++) {
      const f32x4 o = slot[w * kTallTX + tx];
#pragma unroll
      for (int i = 0; i < 4; i++) top[i] = fmaxf(top[i], o[i]);
    }
    parity ^= 1;  // the next tile's maxima go to the other half, so one barrier per tile is enough
    f32x4 sc;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      sc[i] = top[i] / 127.0f;  // the one IEEE divide per channel
      rcp[i] = reciprocal_of(divisor_of(sc[i]));
    }
    if (tx * 4 < width_of(cur) && ty == 0)
      *reinterpret_cast<f32x4*>(scales + (int64_t)cur.slab * D + first_channel_of(cur) + tx * 4) = sc;

    if (ticket) {
      if (tid == 0) {
        const uint32_t all_here = turns * neighbours;
        uint32_t seen = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1;
        for (int poll = 0; seen < all_here && poll < kTallPolls; poll++) {
          __builtin_amdgcn_s_sleep(16);
          seen = __hip_atomic_load(ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      __syncthreads();
    }
  }
  if (ticket && tid == 0 && turns > 0) {
    const uint32_t last = (turns + 1) * neighbours - 1;
    if (__hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == last)
      __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

}  // namespace

// The kernels ask for more dynamic LDS than a kernel gets by default: raise their limits, once per device
// (also from kvq_prepare_stream, so that nothing but launches is left for a stream capture).
kvq_status prepare_fused_tall() {
  static std::atomic<uint64_t> done{0};
  int dev = -1;
  KVQ_HIP(hipGetDevice(&dev));
  const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t)1 << dev : 0;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return KVQ_OK;
#define KVQ_RAISE_LDS(TXLOG_, NT_)                                                                    \
  KVQ_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&fused_tall_kernel<TXLOG_, NT_>),         \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)tall_lds_bytes(1 << TXLOG_)))
  KVQ_RAISE_LDS(3, false);
  KVQ_RAISE_LDS(4, false);
  KVQ_RAISE_LDS(5, false);
  KVQ_RAISE_LDS(5, true);
  KVQ_RAISE_LDS(6, false);
  KVQ_RAISE_LDS(6, true);
#undef KVQ_RAISE_LDS
  if (bit) done.fetch_or(bit, std::memory_order_release);
  return KVQ_OK;
}

// log2 of the lanes along a row: the widest tile (up to 256 channels, no wider than the rows) whose
// 64 rows per lane still reach N
static int tall_tx_log2(int64_t N, int64_t D) {
  int l = 3;
  while (l < 6 && N <= (int64_t)kTallRowsPerLane * (kTallBlock >> (l + 1)) && ((int64_t)4 << l) < D) l++;
  return l;
}

// Whether kvq_quantize_fused gives a problem to these kernels; `slab_form` says that the register-only kernel
// (kvq_fused.hip) could take it too.  The tile has to be more than half full (the arithmetic of a turn is
// that of a full tile), every byte offset inside it has to fit 32 bits, and then, measured
// (profiles/fused_column_tiles.md):
//  - more than 2048 rows (tiles of 32 channels): always -- the register-only kernel has only 16-channel
//    tiles there ([256 x 4096 x 128] 0.143 against 0.162 ms, [2048 x 4096 x 128] 1.22 against 1.30);
//  - 1025 to 2048 rows (tiles of 64 channels): while a compute unit gets fewer than eight tiles --
//    [256 x 2048 x 256] 0.128 against 0.138 ms for the register-only kernel, whose 16 rows per lane leave one
//    workgroup per unit with nothing to overlap, but [2048 x 2048 x 128] 0.605 against 0.582 ms: over many
//    turns the waiting for the neighbour costs more than that;
//  - up to 1024 rows (tiles of 128 or 256 channels): only without the other kernel, which runs two
//    workgroups of 8 rows per lane on a unit there and is level or ahead -- [512 x 1024 x 256] 0.123 against
//    0.137 ms, [512 x 512 x 1024] 0.220 against 0.232, [2048 x 1024 x 128] 0.245 against 0.236.
// KVQ_OPT_FUSED_TALL = 3 takes every problem whose tiles are more than half full.
bool fused_tall_applicable(const float* x, const float* scales, const int8_t* codes, int64_t batch, int64_t N,
                           int64_t D, bool slab_form) {
  const int mode = options().fused_tall;
  if (mode == 0) return false;
  if (D % 4 || !aligned(x, 16) || !aligned(scales, 16) || !aligned(codes, 4)) return false;
  if (N > kTallRowsPerLane * (kTallBlock >> 3) || D > 65536) return false;
  const int tx_log2 = tall_tx_log2(N, D);
  if (2 * N <= (int64_t)kTallRowsPerLane * (kTallBlock >> tx_log2)) return false;
  if (mode == 3 || tx_log2 == 3 || !slab_form) return true;
  if (tx_log2 > 4) return false;
  const int64_t tile_channels = (int64_t)4 << tx_log2;
  return batch * ((D + tile_channels - 1) / tile_channels) < 8 * (int64_t)current_device().cus;
}

kvq_status launch_fused_tall(const float* x, float* scales, int8_t* codes, int64_t batch, int64_t N, int64_t D,
                             const Workspace& ws, hipStream_t stream) {
  const DeviceInfo dev = current_device();
  if (dev.cus <= 0) return hip_failed(hipErrorInvalidDevice);
  if (kvq_status s = prepare_fused_tall()) return s;
  const int tx_log2 = tall_tx_log2(N, D);
  const int64_t tile_channels = (int64_t)4 << tx_log2;
  const int64_t ctiles = (D + tile_channels - 1) / tile_channels;
  // column tiles that share a 128-byte line of codes: four of 32 channels, two of 64, else each has its own
  const int line_log2 = tx_log2 == 3 ? 2 : tx_log2 == 4 ? 1 : 0;
  int quad_log2 = 0;
  while (quad_log2 < line_log2 && ((int64_t)1 << quad_log2) < ctiles) quad_log2++;
  const int64_t quad_tiles = (int64_t)1 << quad_log2;
  const int64_t quads_per_slab = (ctiles + quad_tiles - 1) / quad_tiles;
  if (batch > INT32_MAX / (2 * kTallXcds) / quads_per_slab) return KVQ_ERR_OVERFLOW;
  const int64_t total_quads = batch * quads_per_slab;
  // one workgroup per compute unit, the same number on every XCD and whole quads of them, no more than the
  // longest sequence has tiles; a workgroup then moves on by per_xcd / quad_tiles quads of its XCD a step
  int64_t per_xcd = dev.cus / kTallXcds / quad_tiles * quad_tiles;
  if (per_xcd < quad_tiles) per_xcd = quad_tiles;
  const int64_t longest = (total_quads + kTallXcds - 1) / kTallXcds * quad_tiles;
  if (per_xcd > longest) per_xcd = longest;
  const int64_t step = kTallXcds * (per_xcd / quad_tiles);  // in quads, slab-major
  // a counter per group of neighbours; none where a quad is a single tile or the workspace has too few
  uint32_t* const tickets =
      options().fused_tall != 2 && quad_tiles > 1 && step <= kTickets ? ws.tickets : nullptr;
  // rows of codes that are whole cache lines can be streamed out
  const bool nt = tx_log2 >= 5 && D % 128 == 0 && aligned(codes, 128);
  const dim3 grid((uint32_t)(per_xcd * kTallXcds)), block(kTallBlock);
#define KVQ_LAUNCH_TALL(TXLOG_, NT_)                                                                              \
  hipLaunchKernelGGL((fused_tall_kernel<TXLOG_, NT_>), grid, block, tall_lds_bytes(1 << TXLOG_), stream, x, scales, \
                     codes, (uint32_t)total_quads, (uint32_t)quads_per_slab, (uint32_t)quad_log2,                 \
                     (uint32_t)(step / quads_per_slab), (uint32_t)(step % quads_per_slab), (uint32_t)N,           \
                     (uint32_t)D, tickets)
  if (tx_log2 == 3) KVQ_LAUNCH_TALL(3, false);
  else if (tx_log2 == 4) KVQ_LAUNCH_TALL(4, false);
  else if (tx_log2 == 5 && nt) KVQ_LAUNCH_TALL(5, true);
  else if (tx_log2 == 5) KVQ_LAUNCH_TALL(5, false);
  else if (nt) KVQ_LAUNCH_TALL(6, true);
  else KVQ_LAUNCH_TALL(6, false);
#undef KVQ_LAUNCH_TALL
  KVQ_HIP(hipGetLastError());
  return KVQ_OK;
}

}  // namespace kvq
