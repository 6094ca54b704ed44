/*
 * kvq.h -- C ABI of the MI355X (gfx950) per-channel symmetric INT8 KV-cache
 * quantization library (libkvq.so).
 *
 * Data model (paper, "Data Structures" and "Per-Channel INT8 Quantization"):
 * a key or value matrix is token-major, row-major fp32 [N tokens x D channels]
 * with the channel index contiguous; one fp32 scale per channel (column).  An
 * optional leading `batch` dimension stacks independent [N x D] slabs
 * contiguously (slab stride N*D elements); scales are then [batch x D].  A
 * [B,H,T,d] cache is batch = B*H, N = T, D = d.
 *
 * Conventions for every entry point:
 *  - every data pointer is a DEVICE pointer owned by the caller; the library
 *    never frees or keeps it.  Scalar results are written to device memory too,
 *    so no call synchronises: work is enqueued on `stream` (NULL = the default
 *    stream) and the call returns.
 *  - any N, D, batch >= 1 is accepted.  Rows whose width or base address do not
 *    allow 16-byte vector access take a slower generic kernel with identical
 *    results; nothing is skipped.
 *  - inputs must be finite (no NaN/Inf); subnormals are honoured (no flush).
 *  - argument errors are detected on the host before anything is enqueued and
 *    reported as a negative status with no side effects; a failed HIP call maps
 *    to KVQ_ERR_HIP.  Input and output buffers must not overlap.
 *  - the scale reductions (kvq_absmax_scales and its _t, _int4, _fp8 forms),
 *    kvq_roundtrip_error and kvq_attn_score_error keep a per-device, per-stream
 *    workspace (16 MiB of partial maxima and sums, 4 KiB of counters) that the library allocates with
 *    hipMalloc on a stream's first such call (or in kvq_prepare_stream) and keeps
 *    until kvq_release_stream or the end of the process -- make that call outside
 *    any graph capture.  Two calls in flight on
 *    the SAME stream are ordered by the stream; calls on different streams use
 *    different workspaces.  kvq_append and kvq_quantize_fused run a scale
 *    reduction and so use it too.
 *  - results of kvq_absmax_scales, kvq_quantize, kvq_dequantize are unique bit
 *    patterns; the error statistics are deterministic for a given shape.
 */
#ifndef KVQ_H
#define KVQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int kvq_status;
#define KVQ_OK 0
#define KVQ_ERR_NULL (-1)     /* a required pointer is NULL                               */
#define KVQ_ERR_SHAPE (-2)    /* batch, N, D or Q is < 1                                  */
#define KVQ_ERR_OVERFLOW (-3) /* batch*N*D (or a launch dimension) exceeds what is indexable */
#define KVQ_ERR_HIP (-4)      /* a HIP runtime call failed; see kvq_last_hip_error()      */
#define KVQ_ERR_ARG (-5)      /* inconsistent optional arguments                          */
#define KVQ_ERR_LIMIT (-6)    /* larger than the fixed scratch of an entry point that allocates nothing */

/* Same type as hipStream_t (an opaque pointer); declared here so that callers
 * need no HIP headers. */
typedef struct ihipStream_t *kvq_stream_t;

/*
 * Scale computation -- Eq. (scale)/(scale_compute) and Algorithm "Compute
 * Scales": scales[b,d] = max_t |x[b,t,d]| / 127 (one IEEE fp32 divide), +0 for
 * an all-zero channel.
 *   x      [batch,N,D] fp32, device, read only
 *   scales [batch,D]   fp32, device, written once per channel (4-byte alignment
 *                      suffices); partial maxima live in the stream's workspace
 */
kvq_status kvq_absmax_scales(const float *x, float *scales,
                             int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * kvq_absmax_scales for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same bits
 * as kvq_absmax_scales, but the partial maxima of a reduction split over row chunks go to a fixed
 * array inside the library's device image instead of the per-stream workspace, so this call never
 * calls hipMalloc / hipFree (nor any allocating library routine), on its first use either.
 *   limit: batch * D <= KVQ_STATIC_SCRATCH_FLOATS channels (one slot per channel and row chunk;
 *          8 MiB of device memory that every GPU the library runs on holds until the process
 *          ends).  Beyond it: KVQ_ERR_LIMIT, nothing enqueued.  Within it, fewer slots only mean
 *          fewer, longer row chunks.
 *   sharing: all calls on one GPU use that GPU's one array, whatever their stream.  Calls on the
 *          same stream are ordered by it; calls in flight at the same time on different streams
 *          of one GPU race on the array and give undefined scales.  The array keeps the last
 *          call's contents; nothing in it needs clearing, because each call writes every slot it
 *          later reads.
 */
#define KVQ_STATIC_SCRATCH_FLOATS 2097152
kvq_status kvq_absmax_scales_static(const float *x, float *scales,
                                    int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * Quantization -- Eq. (quantize)/(quant_op) plus the stated clamp:
 * codes[b,t,d] = clamp(rint(x[b,t,d] / scales[b,d]), -127, 127) with a
 * correctly rounded fp32 divide and round-half-to-even; 0 where the scale is 0.
 * Any positive scale is accepted (not only the one kvq_absmax_scales gives).
 *   x [batch,N,D] fp32, scales [batch,D] fp32: device, read only
 *   codes [batch,N,D] int8: device, written
 */
kvq_status kvq_quantize(const float *x, const float *scales, int8_t *codes,
                        int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * Dequantization -- Eq. (dequantize)/(dequant_op):
 * x_hat[b,t,d] = (float)codes[b,t,d] * scales[b,d] (one fp32 multiply).
 *   codes [batch,N,D] int8, scales [batch,D] fp32: device, read only
 *   x_hat [batch,N,D] fp32: device, written
 */
kvq_status kvq_dequantize(const int8_t *codes, const float *scales, float *x_hat,
                          int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * The three calls above for matrices kept in fp16 or bf16 (the formats real caches
 * use; "Memory Bottleneck in LLM Inference").  x / x_hat point to 16-bit elements
 * in the same [batch,N,D] layout.  A 16-bit value widens to fp32 exactly, so scales
 * and codes are those of the widened matrix; dequantization forms (float)code *
 * scale in fp32 and rounds it to nearest even into the 16-bit format.  Scales stay
 * fp32.  dtype KVQ_DTYPE_F32 forwards to the fp32 calls; an unknown dtype or an
 * odd 16-bit pointer gives KVQ_ERR_ARG.
 */
#define KVQ_DTYPE_F32 0
#define KVQ_DTYPE_F16 1
#define KVQ_DTYPE_BF16 2
kvq_status kvq_absmax_scales_t(int dtype, const void *x, float *scales,
                               int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);
kvq_status kvq_quantize_t(int dtype, const void *x, const float *scales, int8_t *codes,
                          int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);
kvq_status kvq_dequantize_t(int dtype, const int8_t *codes, const float *scales, void *x_hat,
                            int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * The same method with 4-bit codes -- Limitations, "Lower bit-widths" (INT4 for 8x
 * compression): the integer range of Eq. (scale) / Eq. (quantize) becomes [-7, 7]:
 *   scales[b,d]  = max_t |x[b,t,d]| / 7
 *   code[b,t,d]  = clamp(rint(x[b,t,d] / scales[b,d]), -7, 7), 0 where the scale is 0
 *   x_hat[b,t,d] = (float)code[b,t,d] * scales[b,d]
 * with the same fp32 divide, rounding and multiply as the 8-bit calls.  Codes are
 * stored two per byte in two's complement, channel 2j in the low nibble and channel
 * 2j+1 in the high nibble of byte j of the row, so D must be even (KVQ_ERR_ARG
 * otherwise) and packed is [batch, N, D/2] bytes.
 *   x / x_hat [batch,N,D] fp32, scales [batch,D] fp32, packed [batch,N,D/2] uint8: device
 */
kvq_status kvq_absmax_scales_int4(const float *x, float *scales,
                                  int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);
kvq_status kvq_quantize_int4(const float *x, const float *scales, uint8_t *packed,
                             int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);
kvq_status kvq_dequantize_int4(const uint8_t *packed, const float *scales, float *x_hat,
                               int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * The same method with FP8 codes -- Future Work ("GPU-specific numeric formats such as
 * FP8").  The 8-bit code is an OCP E4M3 number (1 sign, 4 exponent bits with bias 7, 3
 * mantissa bits, subnormals, largest finite value 448; the NaN patterns 0x7F / 0xFF are
 * never produced) instead of an integer:
 *   scales[b,d]  = max_t |x[b,t,d]| / 448
 *   code[b,t,d]  = E4M3(x[b,t,d] / scales[b,d]): the fp32 quotient (same divide as the int8
 *                  call) rounded to the nearest E4M3 value, ties to the even mantissa,
 *                  saturated at +-448; the sign of the quotient is kept (so -0 exists);
 *                  0x00 where the scale is 0
 *   x_hat[b,t,d] = value(code) * scales[b,d]   (value() exact in fp32, one multiply)
 * Relative error of a reconstructed value is at most 2^-4 (half a mantissa step) down to
 * |x| = scale * 2^-6, against the absolute bound scale/2 of the integer codes.
 *   x / x_hat [batch,N,D] fp32, scales [batch,D] fp32, codes [batch,N,D] uint8: device
 */
kvq_status kvq_absmax_scales_fp8(const float *x, float *scales,
                                 int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);
kvq_status kvq_quantize_fp8(const float *x, const float *scales, uint8_t *codes,
                            int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);
kvq_status kvq_dequantize_fp8(const uint8_t *codes, const float *scales, float *x_hat,
                              int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * Streaming append -- Limitations, "Dynamic quantization" (scales that adapt during
 * inference) and Future Work (streaming workloads), with the operations of Eq. (scale),
 * Eq. (quant_op) and Eq. (dequant_op).  A cache of n_old tokens exists only as int8
 * codes and per-channel scales; m new fp32 tokens join it:
 *   cand[b,d]  = max_t |x_new[b,t,d]| / 127
 *   s_new[b,d] = cand > s_old ? cand : s_old        (so scales track the running absmax)
 *   channels with s_new > s_old, cached tokens t < n_old:
 *       codes[b,t,d] <- clamp(rint(((float)codes[b,t,d] * s_old) / s_new), -127, 127)
 *       (the code is re-expressed from its reconstruction; the fp32 original is gone, so
 *        each growth of a channel can add up to s_new/2 to the error of its cached tokens)
 *   new tokens: codes[b,n_old+t,d] = clamp(rint(x_new[b,t,d] / s_new), -127, 127), 0 if s_new == 0
 * Channels that did not grow keep their codes bit for bit; rows >= n_old + m are not touched.
 *   x_new       [batch,m,D] fp32, device, read only
 *   scales      [batch,D] fp32, device: s_old on entry (all 0 for an empty cache), s_new on return
 *   scales_prev [batch,D] fp32, device, written: s_old (also used as scratch during the call);
 *               must not overlap scales
 *   codes       [batch,capacity,D] int8, device: rows [0,n_old) read and possibly rewritten,
 *               rows [n_old,n_old+m) written
 * n_old >= 0, m >= 1, n_old + m <= capacity (KVQ_ERR_SHAPE / KVQ_ERR_ARG otherwise).
 */
kvq_status kvq_append(const float *x_new, float *scales, float *scales_prev, int8_t *codes,
                      int64_t batch, int64_t n_old, int64_t m, int64_t capacity, int64_t D,
                      kvq_stream_t stream);

/*
 * The same append for new tokens in a 16-bit format ("Memory Bottleneck in LLM Inference":
 * activations and caches are kept in 16-bit formats): x_new [batch,m,D] holds fp16 or bf16
 * values (dtype KVQ_DTYPE_F16 / KVQ_DTYPE_BF16, 2-byte aligned), which widen to fp32 exactly,
 * so scales and codes are those kvq_append gives for the widened tokens.  KVQ_DTYPE_F32
 * forwards to kvq_append; any other dtype is KVQ_ERR_ARG.  All other arguments as above.
 */
kvq_status kvq_append_t(int dtype, const void *x_new, float *scales, float *scales_prev, int8_t *codes,
                        int64_t batch, int64_t n_old, int64_t m, int64_t capacity, int64_t D,
                        kvq_stream_t stream);

/*
 * The same append onto a 4-bit cache (kvq_quantize_int4's packed layout; Limitations, "Lower
 * bit-widths" together with "Dynamic quantization"): the formulas of kvq_append with 127 replaced
 * by 7 -- cand = absmax / 7, codes clamped to [-7, 7], cached codes of grown channels re-expressed
 * from (float)code * s_old -- and two codes per byte.
 *   x_new  [batch,m,D] fp32, device, read only
 *   scales, scales_prev as for kvq_append
 *   packed [batch,capacity,D/2] uint8, device: rows [0,n_old) read and possibly rewritten,
 *          rows [n_old,n_old+m) written, later rows untouched
 * D must be even (KVQ_ERR_ARG); other errors as for kvq_append.
 */
kvq_status kvq_append_int4(const float *x_new, float *scales, float *scales_prev, uint8_t *packed,
                           int64_t batch, int64_t n_old, int64_t m, int64_t capacity, int64_t D,
                           kvq_stream_t stream);

/*
 * Scale computation and quantization in one call -- Eq. (scale_compute) and
 * Eq. (quant_op); same results, bit for bit, as kvq_absmax_scales followed by
 * kvq_quantize.  Slabs of at most 4096 rows (D % 4 == 0, 16-byte aligned x and
 * scales, 4-byte aligned codes) are cut into column tiles that one workgroup
 * holds on chip -- in registers up to 2048 rows, in registers and LDS up to
 * 4096 (D <= 65536 there) -- so x is fetched from HBM once, in one launch.
 * Taller slabs, other widths and other alignments run the two passes back to
 * back.  The form that also uses LDS keeps a few counters in the stream's
 * workspace (see the notes at the top) and leaves them at zero.
 *   x [batch,N,D] fp32 read only; scales [batch,D] fp32 and codes [batch,N,D]
 *   int8 written.  Errors as for kvq_absmax_scales.
 */
kvq_status kvq_quantize_fused(const float *x, float *scales, int8_t *codes,
                              int64_t batch, int64_t N, int64_t D, kvq_stream_t stream);

/*
 * Reconstruction error -- Introduction ("Reconstruction error: L2 error and
 * maximum absolute error") and Evaluation, "Reconstruction Error":
 *   *sumsq_out  = sum over all elements of (x - x_hat)^2   (fp32 difference,
 *                 fp64 square and sum; the L2 error is its square root)
 *   *maxabs_out = max over all elements of |x - x_hat|
 * Two forms:
 *   x_hat != NULL: compare x with the fp32 matrix x_hat (codes, scales ignored,
 *                  may be NULL);
 *   x_hat == NULL: codes and scales are required and x_hat is recomputed on the
 *                  fly as (float)code * scale, bit-identical to kvq_dequantize.
 *   sumsq_out (double, 8-byte aligned) and maxabs_out (float): device, written.
 */
kvq_status kvq_roundtrip_error(const float *x, const float *x_hat,
                               const int8_t *codes, const float *scales,
                               int64_t batch, int64_t N, int64_t D,
                               double *sumsq_out, float *maxabs_out, kvq_stream_t stream);

/*
 * Attention-score error -- Introduction ("mean absolute difference between
 * attention dot products computed with original and reconstructed keys") and
 * Evaluation, "Attention Score Error":
 *   *mean_abs_out = (1/(Q*N)) sum_{j<Q, t<N} | q_j . k_t  -  q_j . k_hat_t |
 * raw dot products (no 1/sqrt(d), no softmax).  Computed as sum_d q_j[d] e_t[d]
 * with e = k - k_hat formed in fp32 (exact there), contracted on the matrix
 * cores in runs of 64 channels that are rounded to fp32 and added up in fp64;
 * absolute value and mean in fp64.  Every score is within
 * 65 * 2^-24 * sum_d |q_j[d] e_t[d]| of the exact one (the errors are centred:
 * the mean moves by far less).  Beyond finite inputs this needs the 64-channel
 * sums of |q e| inside the fp32 range; values of |q| or |e| below 2^-110 may
 * lose low bits.
 *   queries [Q,D] fp32, k [N,D] fp32: device, read only
 *   k_hat [N,D] fp32, or NULL with codes [N,D] int8 + scales [D] fp32 given
 *   (k_hat recomputed as in kvq_dequantize)
 *   mean_abs_out: device double, written.
 */
kvq_status kvq_attn_score_error(const float *queries, int64_t Q,
                                const float *k, const float *k_hat,
                                const int8_t *codes, const float *scales,
                                int64_t N, int64_t D,
                                double *mean_abs_out, kvq_stream_t stream);

/*
 * Attention scores straight from the quantized cache -- Background, Eq. (attention)
 * (the raw dot products q.k, no 1/sqrt(d), no softmax) with k replaced by the
 * reconstruction of Eq. (dequant_op):
 *   scores_out[b,j,t] = sum_d queries[b,j,d] * ((float)codes[b,t,d] * scales[b,d])
 * The scale is folded into the query (qs = q*s, one fp32 rounding) and the codes are
 * used as read.  Two forms, chosen by shape:
 *  - Q >= 3, 16-byte aligned codes, and D % 64 == 0 up to 1024 or D % 256 == 0 up to
 *    8192: int8 matrix cores.  qs is
 *    taken to 28-bit fixed point relative to the largest |qs| of its query, the integer
 *    dot products are exact, the result is rounded once to fp32.  Against exact
 *    arithmetic: 2^-27 * max_d|queries*scales| * sum_d|codes|
 *                + 4 * 2^-24 * sum_d |queries * codes * scales|.
 *    Independent of launch shape and accumulation order.
 *  - otherwise fp32 FMAs: (16*ceil(D/1024) + 12) * 2^-24 * sum_d |queries * codes * scales|
 *    for D % 16 == 0 with 16-byte aligned inputs, (D + 4) * 2^-24 * the same sum for the
 *    generic kernel.
 *  Where q*s or the score falls below 2^-126 (fp32 gradual underflow) add (127 D + 1) * 2^-150.
 *   queries [batch,Q,D] fp32, codes [batch,N,D] int8, scales [batch,D] fp32:
 *   device, read only.  scores_out [batch,Q,N] fp32: device, written.
 * Any Q >= 1; queries per pass over the codes: 8 (fp32 form), 16 / 8 / 4 on the matrix cores for
 * D <= 512 / 1024 / 8192.
 */
kvq_status kvq_scores_from_codes(const float *queries, int64_t Q, const int8_t *codes,
                                 const float *scales, int64_t batch, int64_t N, int64_t D,
                                 float *scores_out, kvq_stream_t stream);

/*
 * kvq_scores_from_codes for a 4-bit cache (kvq_quantize_int4's packed layout, scales =
 * absmax / 7): scores_out[b,j,t] = sum_d queries[b,j,d] * ((float)code[b,t,d] * scales[b,d])
 * with code in [-7, 7].  D must be even (KVQ_ERR_ARG otherwise).  D % 128 == 0, D <= 1024
 * and 16-byte aligned packed rows run on the int8 matrix cores with the error bound of the
 * 8-bit matrix-core form; any other shape takes a scalar fp32 kernel with the bound
 * (D + 4) * 2^-24 * sum_d |queries * codes * scales|.
 *   queries [batch,Q,D] fp32, packed [batch,N,D/2] uint8, scales [batch,D] fp32: device,
 *   read only.  scores_out [batch,Q,N] fp32: device, written.
 */
kvq_status kvq_scores_from_codes_int4(const float *queries, int64_t Q, const uint8_t *packed,
                                      const float *scales, int64_t batch, int64_t N, int64_t D,
                                      float *scores_out, kvq_stream_t stream);

/* Human-readable name of a status code (static string, never NULL). */
const char *kvq_status_string(kvq_status status);

/* The hipError_t value of the last failed HIP call on this thread (0 if none). */
int kvq_last_hip_error(void);

/*
 * Creates the current device's workspace for `stream` now (one hipMalloc; nothing happens if it
 * exists) and does the once-per-device set-up of the score-error kernels (their LDS limit), so that
 * the first reduction on that stream allocates nothing and enqueues nothing but kernels -- call it
 * before capturing a graph on the stream, or before entering a region that must not allocate.
 */
kvq_status kvq_prepare_stream(kvq_stream_t stream);

/*
 * Frees the current device's workspace of `stream` (hipFree, which waits for the device), e.g.
 * before the stream is destroyed.  No library call may be in flight on that stream.  Without
 * this call a workspace lives until the process ends.  KVQ_OK also when there is none.
 */
kvq_status kvq_release_stream(kvq_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_H */
