/*
 * Host logic of libkvq.so under AddressSanitizer and UndefinedBehaviorSanitizer, without a GPU.
 *
 * tests/test_boundary_sanitized.py compiles csrc/kvq_api.hip, kvq_bench.hip and kvq_absmax.hip with the
 * sanitizers on the host side only and loads the result here with lazy binding, so that only what this
 * driver calls has to resolve: argument validation of every entry point (each returns before any HIP
 * call), the launch plans of many shapes, options, status strings.  Undefined arithmetic or a bad
 * access in that host code ends the run with a report.  Prints one line per check group; exit 0 = clean.
 */
#include <dlfcn.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "kvq.h"
#include "kvq_bench.h"

static void *lib;
#define SYM(name) __typeof__(&name) p_##name = (__typeof__(&name))dlsym(lib, #name); \
  if (!p_##name) { fprintf(stderr, "missing symbol %s\n", #name); return 3; }
#define EXPECT(call, want) do { int got_ = (call); if (got_ != (want)) { \
  fprintf(stderr, "line %d: %s gave %d, expected %d\n", __LINE__, #call, got_, (want)); return 1; } } while (0)

int main(int argc, char **argv)
{
    if (argc != 2) return 2;
    lib = dlopen(argv[1], RTLD_LAZY | RTLD_LOCAL);
    if (!lib) { fprintf(stderr, "dlopen: %s\n", dlerror()); return 3; }
    SYM(kvq_plan) SYM(kvq_absmax_scales) SYM(kvq_absmax_scales_static) SYM(kvq_quantize) SYM(kvq_dequantize)
    SYM(kvq_quantize_fused) SYM(kvq_roundtrip_error) SYM(kvq_attn_score_error) SYM(kvq_scores_from_codes)
    SYM(kvq_scores_from_codes_int4) SYM(kvq_append) SYM(kvq_append_t) SYM(kvq_append_int4) SYM(kvq_quantize_int4)
    SYM(kvq_quantize_t) SYM(kvq_quantize_variant) SYM(kvq_probe_stream) SYM(kvq_probe_clock) SYM(kvq_set_option)
    SYM(kvq_get_option) SYM(kvq_status_string)

    float *f = (float *)0x1000;      /* never dereferenced: every call below fails validation first */
    int8_t *c = (int8_t *)0x2000;
    uint8_t *u = (uint8_t *)0x3000;
    double *d = (double *)0x4000;
    const int64_t big = (int64_t)1 << 40, huge = INT64_MAX;

    /* launch plans: a grid of shapes up to the largest sizes, every call, vector and scalar, several CU counts */
    int64_t plan[8];
    long plans = 0;
    const int64_t Ns[] = {1, 2, 63, 64, 65, 1000, 4096, 131072, (int64_t)1 << 21, (int64_t)1 << 31};
    const int64_t Ds[] = {1, 3, 4, 64, 128, 1000, 4100, 8192, (int64_t)1 << 22};
    const int64_t Bs[] = {1, 3, 256, 65536};
    const int cus[] = {1, 104, 256, 65536};
    for (unsigned a = 0; a < sizeof Ns / sizeof *Ns; a++)
        for (unsigned b = 0; b < sizeof Ds / sizeof *Ds; b++)
            for (unsigned e = 0; e < sizeof Bs / sizeof *Bs; e++)
                for (int call = 0; call < 3; call++)
                    for (int vec = 0; vec < 2; vec++)
                        for (unsigned g = 0; g < sizeof cus / sizeof *cus; g++) {
                            const int rc = p_kvq_plan(call, Bs[e], Ns[a], Ds[b], vec, cus[g], plan);
                            if (rc != KVQ_OK && rc != KVQ_ERR_OVERFLOW) {
                                fprintf(stderr, "kvq_plan(%d, %lld, %lld, %lld) gave %d\n", call, (long long)Bs[e],
                                        (long long)Ns[a], (long long)Ds[b], rc);
                                return 1;
                            }
                            if (rc == KVQ_OK && (plan[4] < 1 || plan[5] < 1 || plan[6] < 1)) return 1;
                            plans++;
                        }
    EXPECT(p_kvq_plan(0, huge, huge, huge, 1, 256, plan), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_plan(0, 1, huge, 2, 1, 256, plan), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_plan(9, 1, 8, 8, 1, 256, plan), KVQ_ERR_ARG);
    EXPECT(p_kvq_plan(0, 1, 8, 8, 1, 0, plan), KVQ_ERR_ARG);
    EXPECT(p_kvq_plan(0, 1, 8, 8, 1, 256, NULL), KVQ_ERR_NULL);
    printf("launch plans: %ld computed\n", plans);

    /* argument validation, with sizes at the edge of what 64 bits hold */
    EXPECT(p_kvq_absmax_scales(NULL, f, 1, 4, 4, NULL), KVQ_ERR_NULL);
    EXPECT(p_kvq_absmax_scales(f, f, 0, 4, 4, NULL), KVQ_ERR_SHAPE);
    EXPECT(p_kvq_absmax_scales(f, f, 1, huge, huge, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_absmax_scales(f, f, huge, 1, 1, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_absmax_scales_static(f, f, 1, 4, (int64_t)KVQ_STATIC_SCRATCH_FLOATS + 1, NULL), KVQ_ERR_LIMIT);
    EXPECT(p_kvq_absmax_scales_static(f, f, huge, huge, huge, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_quantize(f, f, NULL, 1, 4, 4, NULL), KVQ_ERR_NULL);
    EXPECT(p_kvq_quantize(f, f, c, 1, big, big, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_quantize(f, f, c, big, big, 2, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_dequantize(c, f, f, 1, -1, 4, NULL), KVQ_ERR_SHAPE);
    EXPECT(p_kvq_quantize_fused(f, NULL, c, 1, 4, 4, NULL), KVQ_ERR_NULL);
    EXPECT(p_kvq_quantize_t(7, f, f, c, 1, 4, 4, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_quantize_t(KVQ_DTYPE_F16, (char *)f + 1, f, c, 1, 4, 4, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_quantize_int4(f, f, u, 1, 4, 5, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_roundtrip_error(f, NULL, NULL, f, 1, 4, 4, d, f, NULL), KVQ_ERR_NULL);
    EXPECT(p_kvq_roundtrip_error(f, f, NULL, NULL, 1, 4, 4, (double *)((char *)d + 4), f, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_roundtrip_error(f, f, NULL, NULL, huge, 2, 2, d, f, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_attn_score_error(f, 0, f, f, NULL, NULL, 4, 4, d, NULL), KVQ_ERR_SHAPE);
    EXPECT(p_kvq_attn_score_error(f, huge, f, f, NULL, NULL, 4, 4, d, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_attn_score_error(f, 2, f, NULL, NULL, NULL, 4, 4, d, NULL), KVQ_ERR_NULL);
    EXPECT(p_kvq_scores_from_codes(f, huge, c, f, 1, 4, 4, f, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_scores_from_codes(f, 2, c, f, big, big, 4, f, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_scores_from_codes_int4(f, 2, u, f, 1, 4, 5, f, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_append(f, f, f + 64, c, 1, -1, 1, 8, 4, NULL), KVQ_ERR_SHAPE);
    EXPECT(p_kvq_append(f, f, f + 64, c, 1, 8, 1, 8, 4, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_append(f, f, f + 64, c, 1, huge - 1, huge - 1, huge, 4, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_append(f, f, f, c, 1, 0, 1, 8, 4, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_append_t(9, f, f, f + 64, c, 1, 0, 1, 8, 4, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_append_int4(f, f, f + 64, u, 1, 0, 1, 8, 5, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_quantize_variant(9, f, f, c, 1, 4, 4, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_probe_stream(7, f, f, c, c, f, 1, 4, 4, NULL), KVQ_ERR_ARG);
    EXPECT(p_kvq_probe_stream(0, f, f, c, c, f, 1, huge, 4, NULL), KVQ_ERR_OVERFLOW);
    EXPECT(p_kvq_probe_clock(NULL, 10, NULL), KVQ_ERR_NULL);
    EXPECT(p_kvq_probe_clock((uint64_t *)d, 2000000, NULL), KVQ_ERR_ARG);
    printf("argument validation: clean\n");

    /* options: every key, in and out of range, and the extremes of int */
    for (int key = -2; key < 16; key++) {
        const int before = p_kvq_get_option(key);
        const int probes[] = {-2147483647 - 1, -1, 0, 1, 3, 4, 8, 64, 65536, 2147483647};
        for (unsigned i = 0; i < sizeof probes / sizeof *probes; i++) {
            const int rc = p_kvq_set_option(key, probes[i]);
            if (rc != KVQ_OK && rc != KVQ_ERR_ARG) return 1;
        }
        if (before != -2147483647 - 1) p_kvq_set_option(key, before);
    }
    for (int s = -8; s <= 1; s++)
        if (!p_kvq_status_string(s) || !strlen(p_kvq_status_string(s))) return 1;
    printf("options and status strings: clean\n");
    return 0;
}
