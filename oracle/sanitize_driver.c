/*
 * sanitize_driver.c -- runs every function of kvq_oracle.c once on inputs read from a file, with every
 * buffer allocated at exactly the size the function's contract states, and writes all results to a file.
 *
 * TEST INFRASTRUCTURE.  Built together with kvq_oracle.c under -fsanitize=address,undefined by
 * tests/test_oracle_sanitized.py: a read or write outside a buffer, a signed overflow, a misaligned
 * or out-of-range conversion in the oracle ends the run with a report and a non-zero status.  The
 * test then compares the output file byte for byte with what the ordinary build of the oracle gives.
 *
 * Input file:  int64 batch, N, D, Q; float x[batch*N*D]; float queries[Q*D]
 * Output file, in this order: scales[batch*D] f32; codes[batch*N*D] i8; x_hat[batch*N*D] f32;
 *   sumsq f64; maxabs f32; attn f64 (slab 0); scores[Q*N] f64 (slab 0); scales7[batch*D] f32;
 *   codes7[batch*N*D] i8; fp8 codes of x / 448-scales [batch*N*D] u8; fp8 x_hat [batch*N*D] f32;
 *   fp8_encode(x)[batch*N*D] u8; fp8_decode of those [batch*N*D] f32
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void kvq_oracle_compute_scales(const float *x, float *scales, int64_t batch, int64_t N, int64_t D);
void kvq_oracle_quantize(const float *x, const float *scales, int8_t *codes, int64_t batch, int64_t N, int64_t D);
void kvq_oracle_dequantize(const int8_t *codes, const float *scales, float *x_hat, int64_t batch, int64_t N, int64_t D);
void kvq_oracle_roundtrip_error(const float *x, const float *x_hat, int64_t count, double *sumsq_out, float *maxabs_out);
void kvq_oracle_attn_score_error(const float *queries, int64_t Q, const float *k, const float *k_hat, int64_t N,
                                 int64_t D, double *mean_abs_out);
void kvq_oracle_scores_from_codes(const float *queries, int64_t Q, const int8_t *codes, const float *scales,
                                  int64_t N, int64_t D, double *out);
void kvq_oracle_compute_scales_q(const float *x, float *scales, int64_t batch, int64_t N, int64_t D, int qmax);
void kvq_oracle_quantize_q(const float *x, const float *scales, int8_t *codes, int64_t batch, int64_t N, int64_t D,
                           int qmax);
void kvq_oracle_fp8_encode(const float *y, uint8_t *codes, int64_t count);
void kvq_oracle_fp8_decode(const uint8_t *codes, float *y, int64_t count);
void kvq_oracle_quantize_fp8(const float *x, const float *scales, uint8_t *codes, int64_t batch, int64_t N, int64_t D);
void kvq_oracle_dequantize_fp8(const uint8_t *codes, const float *scales, float *x_hat, int64_t batch, int64_t N,
                               int64_t D);

static void *need(size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p) {
        fprintf(stderr, "out of memory\n");
        exit(2);
    }
    return p;
}

static void put(FILE *f, const void *p, size_t bytes)
{
    if (fwrite(p, 1, bytes, f) != bytes) {
        fprintf(stderr, "short write\n");
        exit(2);
    }
}

int main(int argc, char **argv)
{
    if (argc != 3) {
        fprintf(stderr, "usage: %s input output\n", argv[0]);
        return 2;
    }
    FILE *in = fopen(argv[1], "rb");
    int64_t dims[4];
    if (!in || fread(dims, sizeof(int64_t), 4, in) != 4)
        return 2;
    const int64_t batch = dims[0], N = dims[1], D = dims[2], Q = dims[3];
    const size_t E = (size_t)(batch * N * D), S = (size_t)(batch * D);
    float *x = need(E * sizeof(float)), *queries = need((size_t)(Q * D) * sizeof(float));
    if (fread(x, sizeof(float), E, in) != E || fread(queries, sizeof(float), (size_t)(Q * D), in) != (size_t)(Q * D))
        return 2;
    fclose(in);
    FILE *out = fopen(argv[2], "wb");
    if (!out)
        return 2;

    float *scales = need(S * sizeof(float));
    kvq_oracle_compute_scales(x, scales, batch, N, D);
    put(out, scales, S * sizeof(float));

    int8_t *codes = need(E);
    kvq_oracle_quantize(x, scales, codes, batch, N, D);
    put(out, codes, E);

    float *x_hat = need(E * sizeof(float));
    kvq_oracle_dequantize(codes, scales, x_hat, batch, N, D);
    put(out, x_hat, E * sizeof(float));

    double *sumsq = need(sizeof(double));
    float *maxabs = need(sizeof(float));
    kvq_oracle_roundtrip_error(x, x_hat, (int64_t)E, sumsq, maxabs);
    put(out, sumsq, sizeof(double));
    put(out, maxabs, sizeof(float));

    double *attn = need(sizeof(double));
    kvq_oracle_attn_score_error(queries, Q, x, x_hat, N, D, attn);
    put(out, attn, sizeof(double));

    double *scores = need((size_t)(Q * N) * sizeof(double));
    kvq_oracle_scores_from_codes(queries, Q, codes, scales, N, D, scores);
    put(out, scores, (size_t)(Q * N) * sizeof(double));

    float *scales7 = need(S * sizeof(float));
    int8_t *codes7 = need(E);
    kvq_oracle_compute_scales_q(x, scales7, batch, N, D, 7);
    kvq_oracle_quantize_q(x, scales7, codes7, batch, N, D, 7);
    put(out, scales7, S * sizeof(float));
    put(out, codes7, E);

    float *scales8 = need(S * sizeof(float));
    uint8_t *c8 = need(E);
    float *xh8 = need(E * sizeof(float));
    kvq_oracle_compute_scales_q(x, scales8, batch, N, D, 448);
    kvq_oracle_quantize_fp8(x, scales8, c8, batch, N, D);
    kvq_oracle_dequantize_fp8(c8, scales8, xh8, batch, N, D);
    put(out, c8, E);
    put(out, xh8, E * sizeof(float));

    uint8_t *enc = need(E);
    float *dec = need(E * sizeof(float));
    kvq_oracle_fp8_encode(x, enc, (int64_t)E);
    kvq_oracle_fp8_decode(enc, dec, (int64_t)E);
    put(out, enc, E);
    put(out, dec, E * sizeof(float));

    fclose(out);
    free(x); free(queries); free(scales); free(codes); free(x_hat); free(sumsq); free(maxabs); free(attn);
    free(scores); free(scales7); free(codes7); free(scales8); free(c8); free(xh8); free(enc); free(dec);
    return 0;
}
