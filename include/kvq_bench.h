/*
 * kvq_bench.h -- measurement and ablation entry points of libkvq.so.
 *
 * Not part of the method's interface (that is kvq.h): no-math streaming probes, the paper's four
 * kernel designs as ablation points, launch-shape options for sweeps, and the host-side launch
 * plan for tests of the host logic.  Same conventions as kvq.h: device pointers, int64 sizes, a
 * stream, negative status codes on argument errors before anything is enqueued.
 */
#ifndef KVQ_BENCH_H
#define KVQ_BENCH_H

#include "kvq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Quantization by one of the four kernel designs the paper compares ("GPU
 * Kernel Variants": naive = one lane per element, tiled = scales staged in
 * LDS, coarsened = one lane per channel walking the tokens, vectorized = four
 * channels per lane), re-written for gfx950 as ablation points, or by the
 * production kernel.  Same arguments and bit-identical codes as kvq_quantize.
 * KVQ_VARIANT_VECTORIZED needs D % 4 == 0 and 16-byte aligned x and scales
 * (KVQ_ERR_ARG otherwise; the paper's version skips a ragged tail instead).
 */
#define KVQ_VARIANT_PRODUCTION 0
#define KVQ_VARIANT_NAIVE 1
#define KVQ_VARIANT_TILED 2
#define KVQ_VARIANT_COARSENED 3
#define KVQ_VARIANT_VECTORIZED 4
kvq_status kvq_quantize_variant(int variant, const float *x, const float *scales, int8_t *codes,
                                int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * Measurement aid: no-math streaming kernels, to find what this GPU's memory
 * system sustains for the library's traffic patterns over a [batch,N,D] problem.
 *   mode 0: read the fp32 matrix src_f32                  (4 B/element; flat one-shot kernel)
 *   mode 1: write the fp32 matrix dst_f32                 (4 B/element; flat one-shot kernel)
 *   mode 2: the quantize kernel with its arithmetic compiled out: reads src_f32 and
 *           scales, writes dst_i8                         (5 B/element)
 *   mode 3: the dequantize kernel likewise: reads src_i8 and scales, writes dst_f32
 * Pointers a mode does not use may be NULL.  D % 4 == 0; fp32 pointers 16-byte and
 * byte pointers 4-byte aligned (KVQ_ERR_ARG otherwise, also when launch options
 * select another kernel shape than the default).  What is written is meaningless.
 */
kvq_status kvq_probe_stream(int mode, const float *src_f32, float *dst_f32,
                            const int8_t *src_i8, int8_t *dst_i8, const float *scales,
                            int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * Shader clock while other work runs: one wavefront spins for about `microseconds` (1 .. 1000000) and
 * reads the shader-clock counter and the constant 100 MHz wall clock at its start and end.
 *   ticks_out  device pointer to 2 uint64, written: [0] shader-clock ticks, [1] wall-clock ticks
 *              (10 ns each) over the same interval; clock in GHz = 0.1 * [0] / [1]
 * Launch it on a second stream next to the kernels whose clock is of interest.
 */
kvq_status kvq_probe_clock(uint64_t *ticks_out, int microseconds, kvq_stream_t stream);

/*
 * Launch-shape knobs for measurement sweeps; results never depend on them.
 * Returns KVQ_OK, or KVQ_ERR_ARG for an unknown key or a value outside the
 * documented range.  Each host thread has its own set of options (initially the defaults): a thread that sweeps them
 * changes the launches it makes itself and nobody else's, and no lock is needed.
 *   KVQ_OPT_CODEC_WIDTH     elements per lane in quantize/dequantize: 4, 8 or 16
 *   KVQ_OPT_CODEC_UNROLL    rows in flight per lane: 1, 2, 4 or 8; 0 = each kernel's default
 *   KVQ_OPT_BLOCKS_PER_CU   target workgroups per compute unit (used by the error reductions,
 *                           and by quantize/dequantize when PASSES_PER_BLOCK is 0): 1..64;
 *                           0 = each kernel's default
 *   KVQ_OPT_NONTEMPORAL     0/1: streaming cache hints on loads and stores
 *   KVQ_OPT_BLOCK_THREADS   workgroup size of quantize/dequantize: 64, 128, 256 or 512;
 *                           0 = each kernel's default
 *   KVQ_OPT_PASSES_PER_BLOCK  passes of (rows per workgroup x unroll) one workgroup of
 *                           quantize/dequantize makes: 1..65536, or 0 = size the grid from
 *                           BLOCKS_PER_CU instead
 *   KVQ_OPT_ABSMAX_UNROLL   rows in flight per lane in the absmax reduction: 4, 8 or 16
 *   KVQ_OPT_ABSMAX_PASSES   as PASSES_PER_BLOCK, for the absmax reduction
 *   KVQ_OPT_ABSMAX_SPAN     16-byte column groups one lane of the absmax reduction owns per
 *                           row (1, 2, 4 or 8; capped so that a workgroup spans at most a row)
 *   KVQ_OPT_ABSMAX_BLOCKS_PER_CU  target workgroups per compute unit of the absmax reduction
 *                           when ABSMAX_PASSES is 0: 1..64
 *   KVQ_OPT_APPEND_BLOCKS_PER_CU  target workgroups per compute unit of the requantization
 *                           pass of kvq_append (its row chunking): 1..1024
 *   KVQ_OPT_FUSED_MIN_LANES narrowest column tile kvq_quantize_fused may cut a slab into, in lanes of
 *                           4 channels along a row (4, 8, 16, 32, ...; default 8 = 128-byte row
 *                           segments of x, 32-byte segments of codes); slabs that would need narrower
 *                           tiles take the two-pass path
 *   KVQ_OPT_FUSED_MAX_ROWS  rows of its tile a lane of that kernel holds in registers: 4, 8 or 16;
 *                           0 = 8 where the tiles stay at least FUSED_MIN_LANES wide, else 16
 *   KVQ_OPT_FUSED_TALL      the persistent single-pass kernel of kvq_quantize_fused (a column tile of 32 to 256
 *                           channels in the registers and LDS of one workgroup per compute unit; slabs of up to
 *                           4096 rows): 1 (default) = where it is the faster form, 0 = never, 2 = as 1 but its
 *                           workgroups do not wait for the neighbours they share lines of codes with, 3 = wherever
 *                           its tiles are more than half full
 *   KVQ_OPT_ATTN_FORM       which matrix cores kvq_attn_score_error contracts on: 0 = bf16 (every operand as
 *                           three bf16 pieces) where the shape allows, else fp32; 1 = fp32 always.  The two
 *                           forms round differently (both within the bound stated in kvq.h)
 */
#define KVQ_OPT_CODEC_WIDTH 1
#define KVQ_OPT_CODEC_UNROLL 2
#define KVQ_OPT_BLOCKS_PER_CU 3
#define KVQ_OPT_NONTEMPORAL 4
#define KVQ_OPT_BLOCK_THREADS 6
#define KVQ_OPT_PASSES_PER_BLOCK 7
#define KVQ_OPT_ABSMAX_UNROLL 8
#define KVQ_OPT_ABSMAX_PASSES 9
#define KVQ_OPT_ABSMAX_SPAN 10
#define KVQ_OPT_ABSMAX_BLOCKS_PER_CU 11
#define KVQ_OPT_APPEND_BLOCKS_PER_CU 12
#define KVQ_OPT_FUSED_MIN_LANES 13
#define KVQ_OPT_FUSED_MAX_ROWS 14
#define KVQ_OPT_ATTN_FORM 15
#define KVQ_OPT_FUSED_TALL 16
/*
 * The launch plan of a streaming call for a shape, computed on the host without touching a
 * device: how scale reduction, quantize or dequantize (fp32 matrices, current options) would
 * cut [batch,N,D] into workgroups on a GPU with `compute_units` units.  For tests of the host
 * logic and for tuning; nothing is launched.
 *   vector_access  nonzero: buffers are taken to be 16-byte aligned (the vector kernels where D
 *                  allows); zero: the scalar kernels
 *   plan_out       HOST pointer to 8 values, written:
 *     [0] V  adjacent channels a lane owns per column group   [1] J  column groups per lane, TX groups
 *     [2] threads per workgroup = TX * TY                           apart (1 except in the reduction)
 *     [3] TX lanes along a row; lane tx of column tile c owns groups (c*J + j)*TX + tx, j < J
 *     [4] column tiles per row   [5] row chunks per slab   [6] rows per chunk (the last may be short)
 *     [7] rows a lane keeps in flight
 *   work items = batch * row chunks * column tiles; item i is column tile i % tiles of row chunk
 *   (i / tiles) % chunks of slab i / (tiles * chunks); lane ty of a workgroup visits rows
 *   r0 + ty, r0 + ty + TY, ... of its chunk.
 * KVQ_ERR_ARG for an unknown call or compute_units outside 1..65536; shape errors as elsewhere.
 */
#define KVQ_PLAN_ABSMAX 0
#define KVQ_PLAN_QUANTIZE 1
#define KVQ_PLAN_DEQUANTIZE 2
kvq_status kvq_plan(int call, int64_t batch, int64_t N, int64_t D, int vector_access, int compute_units,
                    int64_t *plan_out);

kvq_status kvq_set_option(int key, int value);
int kvq_get_option(int key);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_BENCH_H */
