/*
 * kvq_oracle.c -- CPU oracle for per-channel symmetric INT8 KV-cache quantization.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke
 * check and the benchmark's "cpu_baseline" leg may call it.  It shares no code
 * with the HIP library and must never be used as a fallback for it.
 *
 * Every function is the plain definition from the paper written out as nested
 * loops: single thread, no blocking, no vector intrinsics, no reordering.
 * Build with  gcc -O2 -fno-fast-math -ffp-contract=off  so that each fp32
 * operation below is one correctly rounded IEEE-754 operation (no FMA fusion,
 * no reciprocal substitution, gradual underflow kept).
 *
 * Layout everywhere: token-major ("Data Structures" section): a matrix is
 * [N tokens x D channels], row-major, channel index fastest.  An optional
 * leading dimension `batch` stacks independent [N x D] slabs contiguously
 * (batch = B*H for a [B,H,T,d] cache); each slab has its own D scales.
 *
 * Readings of the paper where it is silent or at odds with itself:
 *  - rounding: the CPU listing rounds ties away from zero while every GPU
 *    listing rounds ties to even; the method is taken to be the GPU one, so
 *    rintf() in the default rounding mode is used.
 *  - a channel whose scale is 0 (all entries zero, or absmax so small that
 *    absmax/127 underflows to 0) gets code 0 everywhere instead of 0/0.
 *  - the clamp to [-127,127] is applied to the rounded float before narrowing.
 *  - "L2 error" is the un-normalised Frobenius norm sqrt(sum (x-xhat)^2); the
 *    sum of squares is returned and the caller takes the root.
 *  - attention-score error uses raw dot products (no 1/sqrt(d), no softmax),
 *    averaged over all (query, token) pairs.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (hand-worked examples, exact rational arithmetic, brute force over scales,
 * the paper's printed error figures, closed forms, numpy special cases).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

/* Scale computation: Eq. (scale) s_d = max_t |K[t,d]| / 127 and Algorithm
 * "Compute Scales": running maximum starts at 0, is replaced only on strict
 * '>', and is divided by 127 once at the end. */
void kvq_oracle_compute_scales(const float *x, float *scales,
                               int64_t batch, int64_t N, int64_t D)
{
    for (int64_t b = 0; b < batch; b++) {
        const float *slab = x + (size_t)b * (size_t)N * (size_t)D;
        for (int64_t d = 0; d < D; d++) {
            float max_abs = 0.0f;
            for (int64_t t = 0; t < N; t++) {
                float a = fabsf(slab[(size_t)t * (size_t)D + (size_t)d]);
                if (a > max_abs)
                    max_abs = a;
            }
            scales[(size_t)b * (size_t)D + (size_t)d] = max_abs / 127.0f;
        }
    }
}

/* Quantization: Eq. (quant_op) K_int8[t,d] = round(K[t,d] / s_d), then the
 * clamp to [-127,127] the Method section states.  One fp32 divide, one
 * round-to-nearest-even, one clamp, one narrowing per element. */
void kvq_oracle_quantize(const float *x, const float *scales, int8_t *codes,
                         int64_t batch, int64_t N, int64_t D)
{
    for (int64_t b = 0; b < batch; b++) {
        for (int64_t t = 0; t < N; t++) {
            for (int64_t d = 0; d < D; d++) {
                size_t i = ((size_t)b * (size_t)N + (size_t)t) * (size_t)D + (size_t)d;
                float s = scales[(size_t)b * (size_t)D + (size_t)d];
                int8_t q;
                if (s == 0.0f) {
                    q = 0;
                } else {
                    float r = rintf(x[i] / s);
                    if (r > 127.0f)
                        r = 127.0f;
                    if (r < -127.0f)
                        r = -127.0f;
                    q = (int8_t)(int)r;
                }
                codes[i] = q;
            }
        }
    }
}

/* Dequantization: Eq. (dequant_op) K_hat[t,d] = K_int8[t,d] * s_d, one
 * int->fp32 conversion (exact) and one fp32 multiply. */
void kvq_oracle_dequantize(const int8_t *codes, const float *scales, float *x_hat,
                           int64_t batch, int64_t N, int64_t D)
{
    for (int64_t b = 0; b < batch; b++) {
        for (int64_t t = 0; t < N; t++) {
            for (int64_t d = 0; d < D; d++) {
                size_t i = ((size_t)b * (size_t)N + (size_t)t) * (size_t)D + (size_t)d;
                float s = scales[(size_t)b * (size_t)D + (size_t)d];
                x_hat[i] = (float)codes[i] * s;
            }
        }
    }
}

/* Reconstruction error (Introduction, "Reconstruction error"; Evaluation,
 * "Reconstruction Error"): the difference is taken in fp32 as the matrices are
 * fp32, its square is accumulated in fp64 over all elements (the L2 error is
 * the root of that sum), and the largest |difference| is the max-abs error. */
void kvq_oracle_roundtrip_error(const float *x, const float *x_hat, int64_t count,
                                double *sumsq_out, float *maxabs_out)
{
    double sumsq = 0.0;
    float maxabs = 0.0f;
    for (int64_t i = 0; i < count; i++) {
        float e = x[i] - x_hat[i];
        sumsq += (double)e * (double)e;
        float a = fabsf(e);
        if (a > maxabs)
            maxabs = a;
    }
    *sumsq_out = sumsq;
    *maxabs_out = maxabs;
}

/* Attention-score error (Introduction, "Attention score error"): for every
 * query j and token t the two dot products q_j.k_t and q_j.k_hat_t are formed
 * (fp64 accumulation), and the absolute differences are averaged over all
 * Q*N pairs. */
void kvq_oracle_attn_score_error(const float *queries, int64_t Q,
                                 const float *k, const float *k_hat,
                                 int64_t N, int64_t D, double *mean_abs_out)
{
    double total = 0.0;
    for (int64_t j = 0; j < Q; j++) {
        const float *q = queries + (size_t)j * (size_t)D;
        for (int64_t t = 0; t < N; t++) {
            const float *kr = k + (size_t)t * (size_t)D;
            const float *hr = k_hat + (size_t)t * (size_t)D;
            double a = 0.0, b = 0.0;
            for (int64_t d = 0; d < D; d++) {
                a += (double)q[d] * (double)kr[d];
                b += (double)q[d] * (double)hr[d];
            }
            total += fabs(a - b);
        }
    }
    *mean_abs_out = total / ((double)Q * (double)N);
}

/* Attention scores straight from the quantized cache (Background, Eq. (attention): the scores are
 * the dot products q.k, here with k replaced by its reconstruction of Eq. (dequant_op)):
 * out[j,t] = sum_d q[j,d] * k_hat[t,d],  k_hat[t,d] = (float)codes[t,d] * scales[d] formed in fp32
 * exactly as dequantization forms it, the dot product accumulated in fp64.  Raw dot products: no
 * 1/sqrt(d) factor and no softmax. */
void kvq_oracle_scores_from_codes(const float *queries, int64_t Q,
                                  const int8_t *codes, const float *scales,
                                  int64_t N, int64_t D, double *out)
{
    for (int64_t j = 0; j < Q; j++) {
        const float *q = queries + (size_t)j * (size_t)D;
        for (int64_t t = 0; t < N; t++) {
            const int8_t *c = codes + (size_t)t * (size_t)D;
            double a = 0.0;
            for (int64_t d = 0; d < D; d++) {
                float k_hat = (float)c[d] * scales[d];
                a += (double)q[d] * (double)k_hat;
            }
            out[(size_t)j * (size_t)N + (size_t)t] = a;
        }
    }
}

/* The same method at another bit width (Limitations, "Lower bit-widths: INT4 ..."): the integer
 * range [-127, 127] of Eq. (scale) / Eq. (quant_op) becomes [-qmax, qmax] (qmax = 7 for 4 bits):
 * scale = absmax / qmax, code = clamp(rint(x / scale), -qmax, qmax).  Codes are returned one per
 * int8; packing two 4-bit codes into a byte is a storage matter done outside the oracle's C code. */
void kvq_oracle_compute_scales_q(const float *x, float *scales, int64_t batch, int64_t N, int64_t D, int qmax)
{
    const float qm = (float)qmax;
    for (int64_t b = 0; b < batch; b++) {
        const float *slab = x + (size_t)b * (size_t)N * (size_t)D;
        for (int64_t d = 0; d < D; d++) {
            float max_abs = 0.0f;
            for (int64_t t = 0; t < N; t++) {
                float a = fabsf(slab[(size_t)t * (size_t)D + (size_t)d]);
                if (a > max_abs)
                    max_abs = a;
            }
            scales[(size_t)b * (size_t)D + (size_t)d] = max_abs / qm;
        }
    }
}

void kvq_oracle_quantize_q(const float *x, const float *scales, int8_t *codes,
                           int64_t batch, int64_t N, int64_t D, int qmax)
{
    const float qm = (float)qmax;
    for (int64_t b = 0; b < batch; b++) {
        for (int64_t t = 0; t < N; t++) {
            for (int64_t d = 0; d < D; d++) {
                size_t i = ((size_t)b * (size_t)N + (size_t)t) * (size_t)D + (size_t)d;
                float s = scales[(size_t)b * (size_t)D + (size_t)d];
                int8_t q = 0;
                if (s != 0.0f) {
                    float r = rintf(x[i] / s);
                    if (r > qm)
                        r = qm;
                    if (r < -qm)
                        r = -qm;
                    q = (int8_t)(int)r;
                }
                codes[i] = q;
            }
        }
    }
}

/* FP8 codes (Future Work: "GPU-specific numeric formats such as FP8"): the per-channel scheme with
 * the 8-bit code an OCP E4M3 floating-point number (1 sign, 4 exponent bits with bias 7, 3 mantissa
 * bits; largest finite value 448; the all-ones pattern is NaN and is never produced) instead of an
 * integer:  scale = absmax / 448,  code = E4M3(x / scale) rounded to nearest even and saturated at
 * +-448,  x_hat = value(code) * scale.  A zero scale gives code 0. */
static uint8_t e4m3_from_float(float y)
{
    uint8_t sign = signbit(y) ? 0x80 : 0x00;
    float a = fabsf(y);
    if (!(a < 448.0f))
        return sign | 0x7E;                      /* 448 and everything above saturates */
    if (a < 0.015625f) {                         /* below 2^-6: multiples of 2^-9 */
        int q = (int)rintf(a * 512.0f);          /* exact scaling; 8 is 2^-6, the smallest normal */
        return sign | (uint8_t)q;
    }
    int e;
    float m = frexpf(a, &e);                     /* a = m * 2^e, m in [0.5, 1) */
    int idx = (int)rintf((m * 2.0f - 1.0f) * 8.0f); /* exact operand; ties to even */
    e -= 1;                                      /* a = (1 + f) * 2^e */
    if (idx == 8) {
        idx = 0;
        e += 1;
    }
    return sign | (uint8_t)(((e + 7) << 3) | idx);
}

static float e4m3_to_float(uint8_t c)
{
    int E = (c >> 3) & 15, M = c & 7;
    float v = E ? ldexpf(1.0f + (float)M / 8.0f, E - 7) : ldexpf((float)M, -9);
    return (c & 0x80) ? -v : v;
}

void kvq_oracle_fp8_encode(const float *y, uint8_t *codes, int64_t count)
{
    for (int64_t i = 0; i < count; i++)
        codes[i] = e4m3_from_float(y[i]);
}

void kvq_oracle_fp8_decode(const uint8_t *codes, float *y, int64_t count)
{
    for (int64_t i = 0; i < count; i++)
        y[i] = e4m3_to_float(codes[i]);
}

void kvq_oracle_quantize_fp8(const float *x, const float *scales, uint8_t *codes,
                             int64_t batch, int64_t N, int64_t D)
{
    for (int64_t b = 0; b < batch; b++)
        for (int64_t t = 0; t < N; t++)
            for (int64_t d = 0; d < D; d++) {
                size_t i = ((size_t)b * (size_t)N + (size_t)t) * (size_t)D + (size_t)d;
                float s = scales[(size_t)b * (size_t)D + (size_t)d];
                codes[i] = s != 0.0f ? e4m3_from_float(x[i] / s) : 0;
            }
}

void kvq_oracle_dequantize_fp8(const uint8_t *codes, const float *scales, float *x_hat,
                               int64_t batch, int64_t N, int64_t D)
{
    for (int64_t b = 0; b < batch; b++)
        for (int64_t t = 0; t < N; t++)
            for (int64_t d = 0; d < D; d++) {
                size_t i = ((size_t)b * (size_t)N + (size_t)t) * (size_t)D + (size_t)d;
                x_hat[i] = e4m3_to_float(codes[i]) * scales[(size_t)b * (size_t)D + (size_t)d];
            }
}
