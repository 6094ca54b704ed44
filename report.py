"""Times every entry point of libkvq.so on each of the five configurations and prints a markdown table.

Usage:  python report.py [--configs 1,2,3,4,5] [--iters 20]
        python report.py --sixteen          (fp16 / bf16 matrices)
        python report.py --int4             (4-bit codes, two per byte)
        python report.py --append           (streaming append onto an int8 cache)
        python report.py --graph            (small configurations: eager launches vs one HIP graph)
        python report.py --fp8              (FP8 E4M3 codes)
        python report.py --scores-int4      (attention scores straight from a 4-bit cache)
        python report.py --scores           (attention scores straight from int8 codes)
        python report.py --attn             (attention-score error over shapes and query counts)
        python report.py --fused            (kvq_quantize_fused against the two calls, by column-tile width;
                                             with --calibration-copy a plain copy of known size is appended
                                             for scaling rocprofv3 --pmc counters)
        python report.py --paper-sweep      (the paper's eight shapes, uniform fills in
                                                                  [-1, 1], its four kernel designs next to
                                                                  the production kernel, and its two error
                                                                  figures computed on the GPU)
Inputs are the seeded synthetic workloads, resident in HBM before timing; times are per launch, from HIP
events around `iters` bursts of 4 back-to-back launches on torch's current stream (mean and fastest burst).
"""
import argparse
import sys

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="1,2,3,4,5")
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--paper-sweep", action="store_true")
    ap.add_argument("--sixteen", action="store_true", help="fp16 / bf16 matrices: absmax, quantize, dequantize")
    ap.add_argument("--int4", action="store_true", help="4-bit codes: absmax, quantize, dequantize, max-abs error")
    ap.add_argument("--append", action="store_true", help="kvq_append: decode steps and prefill chunks")
    ap.add_argument("--graph", action="store_true", help="launch-bound configurations: eager step vs graph replay")
    ap.add_argument("--fp8", action="store_true", help="FP8 (E4M3) codes: absmax, quantize, dequantize, errors")
    ap.add_argument("--scores-int4", action="store_true", help="kvq_scores_from_codes_int4 on decode-like shapes")
    ap.add_argument("--scores", action="store_true", help="kvq_scores_from_codes on decode-like shapes")
    ap.add_argument("--fused", action="store_true", help="kvq_quantize_fused by column-tile width vs two passes")
    ap.add_argument("--attn", action="store_true", help="kvq_attn_score_error over shapes and query counts, both forms")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="with --fused: end with one plain 512 MiB device copy (known traffic for --pmc scaling)")
    args = ap.parse_args()
    import torch
    from paper_2601_04719_amd import kvq, workloads as W

    stream = torch.cuda.current_stream()

    def timeit(f, burst=4):
        # the first tens of milliseconds after an idle phase run at ramping clocks: warm up by time
        import time
        t_end = time.perf_counter() + 0.06
        while time.perf_counter() < t_end:
            for _ in range(5):
                f()
            torch.cuda.synchronize()
        # an event pair around every burst of 4 back-to-back launches: recording an event between two kernels
        # costs a few microseconds of idle GPU, which is 3-4 % of a 0.1 ms kernel
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.iters + 1)]
        ev[0].record(stream)
        for i in range(args.iters):
            for _ in range(burst):
                f()
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        t = [ev[i].elapsed_time(ev[i + 1]) / burst for i in range(args.iters)]
        return float(np.mean(t)), float(np.min(t))

    if args.fused and args.iters == 0:
        # for rocprofv3 --pmc: exactly one launch of each form, in this order, then a plain copy of known size
        kvq.kvq_prepare_stream()
        saved = kvq.kvq_get_option(kvq.OPT_FUSED_MIN_LANES), kvq.kvq_get_option(kvq.OPT_FUSED_TALL)
        for (B, N, D, lanes, tall) in [(256, 4096, 128, 8, 1), (256, 4096, 128, 8, 2), (256, 4096, 128, 4, 0),
                                       (2048, 4096, 128, 8, 1), (2048, 4096, 128, 8, 2), (256, 2048, 256, 8, 1), (256, 2048, 256, 8, 0),
                                       (512, 1024, 256, 8, 1), (4096, 512, 128, 8, 1)]:
            E = B * N * D
            x = torch.randn(E, device="cuda")
            scales = torch.empty(B * D, device="cuda")
            codes = torch.empty(E, dtype=torch.int8, device="cuda")
            torch.cuda.synchronize()
            kvq.kvq_set_option(kvq.OPT_FUSED_MIN_LANES, lanes)
            kvq.kvq_set_option(kvq.OPT_FUSED_TALL, tall)
            kvq.kvq_quantize_fused(x, scales, codes, B, N, D)
            kvq.kvq_set_option(kvq.OPT_FUSED_MIN_LANES, saved[0])
            kvq.kvq_set_option(kvq.OPT_FUSED_TALL, saved[1])
            kvq.kvq_absmax_scales(x, scales, B, N, D)
            kvq.kvq_quantize(x, scales, codes, B, N, D)
            torch.cuda.synchronize()
            print("launched: fused with tiles of >= %d lanes, FUSED_TALL = %d, then the two calls, on [%d x %d x %d]"
                  % (lanes, tall, B, N, D))
            del x, codes
            torch.cuda.empty_cache()
        a = torch.empty(1 << 27, device="cuda")
        b = torch.empty(1 << 27, device="cuda")
        b.copy_(a)
        torch.cuda.synchronize()
        return

    if args.fused:
        print("The register-only kernel by rows per lane and narrowest tile (fused_slab_kernel; the persistent kernel switched off except in the default column):")
        print()
        print("| batch x N x D | two calls ms | fused (default) ms | 16 rows/lane, tiles >= 8 lanes | 16 rows, >= 4 lanes | 8 rows, >= 8 lanes | 8 rows, >= 4 lanes | 4 rows, >= 4 lanes |")
        print("|---|---|---|---|---|---|---|---|")
        saved = kvq.kvq_get_option(kvq.OPT_FUSED_MIN_LANES), kvq.kvq_get_option(kvq.OPT_FUSED_MAX_ROWS)
        for (B, N, D) in [(256, 4096, 128), (256, 2048, 256), (512, 1024, 256), (64, 1024, 2048), (4096, 512, 128),
                          (8192, 256, 128), (1, 1024, 64)]:
            E = B * N * D
            x = torch.randn(E, device="cuda")
            scales = torch.empty(B * D, device="cuda")
            codes = torch.empty(E, dtype=torch.int8, device="cuda")
            two, _ = timeit(lambda: (kvq.kvq_absmax_scales(x, scales, B, N, D), kvq.kvq_quantize(x, scales, codes, B, N, D)))
            cells = []
            tall0 = kvq.kvq_get_option(kvq.OPT_FUSED_TALL)
            for i, (lanes, rows) in enumerate((saved, (8, 16), (4, 16), (8, 8), (4, 8), (4, 4))):
                kvq.kvq_set_option(kvq.OPT_FUSED_MIN_LANES, lanes)
                kvq.kvq_set_option(kvq.OPT_FUSED_MAX_ROWS, rows)
                kvq.kvq_set_option(kvq.OPT_FUSED_TALL, tall0 if i == 0 else 0)  # the other columns: this kernel's forms only
                t, _ = timeit(lambda: kvq.kvq_quantize_fused(x, scales, codes, B, N, D))
                cells.append("%.4f (%.3f)" % (t, 5.0 * E / t / 1e6 / 8000.0))
            kvq.kvq_set_option(kvq.OPT_FUSED_MIN_LANES, saved[0])
            kvq.kvq_set_option(kvq.OPT_FUSED_MAX_ROWS, saved[1])
            kvq.kvq_set_option(kvq.OPT_FUSED_TALL, tall0)
            print("| %d x %d x %d | %.4f | %s |" % (B, N, D, two, " | ".join(cells)))
            sys.stdout.flush()
            del x, codes
            torch.cuda.empty_cache()
        print()
        print("(in brackets: fraction of 8 TB/s at 5 B per element; a setting whose tiles do not fit falls back to the two calls)")
        print()
        print("The persistent kernel (a column tile of 32 to 256 channels in the registers and LDS of one workgroup per compute unit):")
        print()
        print("| batch x N x D | two calls ms | fused (default) ms | its workgroups do not wait for their neighbours | wherever its tiles are at least half full | never (register-only kernel; above 2048 rows its tiles are 16 channels) |")
        print("|---|---|---|---|---|---|")
        saved_tall = kvq.kvq_get_option(kvq.OPT_FUSED_TALL)
        for (B, N, D) in [(256, 4096, 128), (512, 4096, 128), (2048, 4096, 128), (64, 4096, 512), (256, 3072, 128),
                          (1024, 2304, 256), (256, 2048, 256), (512, 2048, 128), (2048, 2048, 128), (512, 1024, 256),
                          (2048, 1024, 128), (512, 512, 1024)]:
            E = B * N * D
            x = torch.randn(E, device="cuda")
            scales = torch.empty(B * D, device="cuda")
            codes = torch.empty(E, dtype=torch.int8, device="cuda")
            two, _ = timeit(lambda: (kvq.kvq_absmax_scales(x, scales, B, N, D), kvq.kvq_quantize(x, scales, codes, B, N, D)))
            cells = []
            # the register-only kernel reaches more than 2048 rows only with tiles of 4 lanes (16 channels)
            for tall, lanes in ((saved_tall, saved[0]), (2, saved[0]), (3, saved[0]), (0, 4 if N > 2048 else saved[0])):
                kvq.kvq_set_option(kvq.OPT_FUSED_TALL, tall)
                kvq.kvq_set_option(kvq.OPT_FUSED_MIN_LANES, lanes)
                kvq.kvq_set_option(kvq.OPT_FUSED_MAX_ROWS, 16 if (tall == 0 and N > 2048) else saved[1])
                t, _ = timeit(lambda: kvq.kvq_quantize_fused(x, scales, codes, B, N, D))
                cells.append("%.4f (%.3f)" % (t, 5.0 * E / t / 1e6 / 8000.0))
            kvq.kvq_set_option(kvq.OPT_FUSED_TALL, saved_tall)
            kvq.kvq_set_option(kvq.OPT_FUSED_MIN_LANES, saved[0])
            kvq.kvq_set_option(kvq.OPT_FUSED_MAX_ROWS, saved[1])
            print("| %d x %d x %d | %.4f | %s |" % (B, N, D, two, " | ".join(cells)))
            sys.stdout.flush()
            del x, codes
            torch.cuda.empty_cache()
        if args.calibration_copy:
            a = torch.empty(1 << 27, device="cuda")
            b = torch.empty(1 << 27, device="cuda")
            b.copy_(a)
            torch.cuda.synchronize()
        return

    if args.sixteen:
        print("| format | batch x N x D | absmax ms (GB/s, of 8 TB/s) | quantize ms (GB/s, of 8 TB/s) | dequantize ms (GB/s, of 8 TB/s) |")
        print("|---|---|---|---|---|")
        for (B, N, D) in [(1, 131072, 8192), (1, 16384, 8192), (256, 4096, 128), (2048, 4096, 128)]:
            E = B * N * D
            for name, dt, tdt in (("fp16", kvq.DTYPE_F16, torch.float16), ("bf16", kvq.DTYPE_BF16, torch.bfloat16)):
                x = torch.randn(E, device="cuda").to(tdt)
                scales = torch.empty(B * D, device="cuda")
                codes = torch.empty(E, dtype=torch.int8, device="cuda")
                xh = torch.empty(E, dtype=tdt, device="cuda")
                ta, _ = timeit(lambda: kvq.kvq_absmax_scales_t(dt, x, scales, B, N, D))
                tq, _ = timeit(lambda: kvq.kvq_quantize_t(dt, x, scales, codes, B, N, D))
                td, _ = timeit(lambda: kvq.kvq_dequantize_t(dt, codes, scales, xh, B, N, D))
                cell = lambda t, bpe: "%.4f (%.0f, %.3f)" % (t, bpe * E / t / 1e6, bpe * E / t / 1e6 / 8000.0)
                print("| %s | %d x %d x %d | %s | %s | %s |" % (name, B, N, D, cell(ta, 2.0), cell(tq, 3.0), cell(td, 3.0)))
                sys.stdout.flush()
                del x, xh, codes
                torch.cuda.empty_cache()
        return

    if args.graph:
        print("| workload | step | launches | eager ms | graph replay ms |")
        print("|---|---|---|---|---|")
        side = torch.cuda.Stream()
        for cfg in (1, 2):
            c = W.CONFIGS[cfg]
            B, N, D, E = c.batch, c.N, c.D, c.elements
            x = torch.from_numpy(W.generate(cfg)).cuda().reshape(-1)
            scales = torch.empty(B * D, device="cuda")
            codes = torch.empty(E, dtype=torch.int8, device="cuda")
            xh = torch.empty(E, device="cuda")
            sumsq = torch.zeros(1, dtype=torch.float64, device="cuda")
            maxabs = torch.zeros(1, device="cuda")

            def step():
                kvq.kvq_absmax_scales(x, scales, B, N, D)
                kvq.kvq_quantize(x, scales, codes, B, N, D)
                kvq.kvq_dequantize(codes, scales, xh, B, N, D)
                kvq.kvq_roundtrip_error(x, xh, None, None, B, N, D, sumsq, maxabs)

            with torch.cuda.stream(side):
                step()
            side.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
            te, _ = timeit(step)
            tg, _ = timeit(graph.replay)
            print("| %s | absmax_scales + quantize + dequantize + roundtrip_error | 7 | %.4f | %.4f |" % (c.name, te, tg))
            sys.stdout.flush()
        return

    if args.append:
        print("| cache batch x capacity x D | new tokens m | token format | slabs (batch > 1) or channels (batch = 1) "
              "that grow | channels grown | mean ms | min ms |")
        print("|---|---|---|---|---|---|---|")
        for (B, cap, D, m, fmt) in [(2048, 4096, 128, 1, "fp32"), (256, 4096, 128, 1, "fp32"),
                                    (32, 131072, 128, 1, "fp32"), (1, 131072, 8192, 1, "fp32"),
                                    (2048, 4096, 128, 16, "fp32"), (2048, 4096, 128, 512, "fp32"),
                                    (1, 131072, 8192, 1024, "fp32"), (2048, 4096, 128, 1, "bf16"),
                                    (2048, 4096, 128, 512, "bf16"), (1, 131072, 8192, 1024, "bf16"),
                                    (2048, 4096, 128, 1, "fp32 onto 4-bit"), (2048, 4096, 128, 512, "fp32 onto 4-bit")]:
            n_old = cap - m
            four = fmt.endswith("4-bit")
            qmax = 7 if four else 127
            if four:
                codes = torch.randint(0, 256, (B * cap * D // 2,), dtype=torch.uint8, device="cuda")
            else:
                codes = torch.randint(-127, 128, (B * cap * D,), dtype=torch.int8, device="cuda")
            scales0 = torch.rand(B * D, device="cuda") + 1.0
            scales = scales0.clone()
            prev = torch.empty_like(scales)
            for frac in (0.0, 0.01, 1.0):
                # new tokens stay inside half the current range; in a fraction of the slabs (of the channels
                # when there is one slab) they reach twice the range, so those scales grow
                x = (torch.rand(B, m, D, device="cuda") - 0.5) * qmax * scales0.view(B, 1, D)
                if frac > 0:
                    if B > 1:
                        x[:max(1, int(round(frac * B)))] *= 4
                    else:
                        x[:, :, :max(1, int(frac * D))] *= 4
                x = x.contiguous()
                if fmt == "bf16":
                    x = x.to(torch.bfloat16)

                def step():
                    scales.copy_(scales0)          # every timed call starts from the same cache state
                    if fmt == "bf16":
                        kvq.kvq_append_t(kvq.DTYPE_BF16, x, scales, prev, codes, B, n_old, m, cap, D)
                    elif four:
                        kvq.kvq_append_int4(x, scales, prev, codes, B, n_old, m, cap, D)
                    else:
                        kvq.kvq_append(x, scales, prev, codes, B, n_old, m, cap, D)

                mean, mn = timeit(step)
                tc, _ = timeit(lambda: scales.copy_(scales0))
                step()
                grown = int((scales > scales0).sum().item())
                print("| %d x %d x %d | %d | %s | %.0f %% | %d | %.4f | %.4f |" % (B, cap, D, m, fmt, 100 * frac, grown,
                                                                                mean - tc, mn - tc))
                sys.stdout.flush()
            del codes
            torch.cuda.empty_cache()
        return

    if args.fp8:
        print("| workload | absmax/448 ms (GB/s, of 8 TB/s) | quantize ms (GB/s, of 8 TB/s) | dequantize ms (GB/s, of 8 TB/s) "
              "| L2 error fp8 | L2 error int8 | max-abs error fp8 | max-abs error int8 |")
        print("|---|---|---|---|---|---|---|---|")
        sumsq = torch.zeros(1, dtype=torch.float64, device="cuda")
        maxabs = torch.zeros(1, dtype=torch.float32, device="cuda")
        for cfg in [int(c) for c in args.configs.split(",")]:
            c = W.CONFIGS[cfg]
            B, N, D, E = c.batch, c.N, c.D, c.elements
            x = torch.from_numpy(W.generate(cfg)).cuda().reshape(-1)
            scales = torch.empty(B * D, device="cuda")
            codes = torch.empty(E, dtype=torch.uint8, device="cuda")
            xh = torch.empty(E, device="cuda")
            ta, _ = timeit(lambda: kvq.kvq_absmax_scales_fp8(x, scales, B, N, D))
            tq, _ = timeit(lambda: kvq.kvq_quantize_fp8(x, scales, codes, B, N, D))
            td, _ = timeit(lambda: kvq.kvq_dequantize_fp8(codes, scales, xh, B, N, D))
            kvq.kvq_roundtrip_error(x, xh, None, None, B, N, D, sumsq, maxabs)
            l8, m8 = float(sumsq.item()) ** 0.5, float(maxabs.item())
            icodes = codes.view(torch.int8)
            kvq.kvq_absmax_scales(x, scales, B, N, D)
            kvq.kvq_quantize(x, scales, icodes, B, N, D)
            kvq.kvq_roundtrip_error(x, None, icodes, scales, B, N, D, sumsq, maxabs)
            li, mi = float(sumsq.item()) ** 0.5, float(maxabs.item())
            cell = lambda t, bpe: "%.4f (%.0f, %.3f)" % (t, bpe * E / t / 1e6, bpe * E / t / 1e6 / 8000.0)
            print("| %s | %s | %s | %s | %.4g | %.4g | %.4g | %.4g |" % (c.name, cell(ta, 4.0), cell(tq, 5.0), cell(td, 5.0),
                                                                        l8, li, m8, mi))
            sys.stdout.flush()
            del x, xh, codes
            torch.cuda.empty_cache()
        return

    if args.int4:
        print("| workload | absmax/7 ms (GB/s, of 8 TB/s) | quantize ms (GB/s, of 8 TB/s) | dequantize ms (GB/s, of 8 TB/s) "
              "| max-abs error 4-bit | max-abs error 8-bit |")
        print("|---|---|---|---|---|---|")
        sumsq = torch.zeros(1, dtype=torch.float64, device="cuda")
        maxabs = torch.zeros(1, dtype=torch.float32, device="cuda")
        for cfg in [int(c) for c in args.configs.split(",")]:
            c = W.CONFIGS[cfg]
            B, N, D, E = c.batch, c.N, c.D, c.elements
            x = torch.from_numpy(W.generate(cfg)).cuda().reshape(-1)
            scales = torch.empty(B * D, device="cuda")
            packed = torch.empty(E // 2, dtype=torch.uint8, device="cuda")
            xh = torch.empty(E, device="cuda")
            ta, _ = timeit(lambda: kvq.kvq_absmax_scales_int4(x, scales, B, N, D))
            tq, _ = timeit(lambda: kvq.kvq_quantize_int4(x, scales, packed, B, N, D))
            td, _ = timeit(lambda: kvq.kvq_dequantize_int4(packed, scales, xh, B, N, D))
            kvq.kvq_roundtrip_error(x, xh, None, None, B, N, D, sumsq, maxabs)
            e4 = float(maxabs.item())
            codes = torch.empty(E, dtype=torch.int8, device="cuda")
            kvq.kvq_absmax_scales(x, scales, B, N, D)
            kvq.kvq_quantize(x, scales, codes, B, N, D)
            kvq.kvq_roundtrip_error(x, None, codes, scales, B, N, D, sumsq, maxabs)
            e8 = float(maxabs.item())
            cell = lambda t, bpe: "%.4f (%.0f, %.3f)" % (t, bpe * E / t / 1e6, bpe * E / t / 1e6 / 8000.0)
            print("| %s | %s | %s | %s | %.4g | %.4g |" % (c.name, cell(ta, 4.0), cell(tq, 4.5), cell(td, 4.5), e4, e8))
            sys.stdout.flush()
            del x, xh, packed, codes
            torch.cuda.empty_cache()
        return

    if args.scores_int4:
        print("| batch x N x D | Q | mean ms | bytes moved (GB) | GB/s | of 8 TB/s | tokens scored per second (G) |")
        print("|---|---|---|---|---|---|---|")
        for (B, N, D) in [(256, 4096, 128), (2048, 4096, 128), (32, 131072, 128), (512, 4096, 256)]:
            E = B * N * D
            packed = torch.randint(0, 256, (E // 2,), dtype=torch.uint8, device="cuda")
            scales = torch.rand(B * D, device="cuda") + 0.1
            for Q in (1, 2, 4, 8, 16):
                q = torch.randn(B * Q * D, device="cuda")
                out = torch.empty(B * Q * N, device="cuda")
                m, _ = timeit(lambda: kvq.kvq_scores_from_codes_int4(q, Q, packed, scales, B, N, D, out))
                nbytes = E / 2 + 4.0 * B * Q * N + 4.0 * B * Q * D + 4.0 * B * D
                print("| %d x %d x %d | %d | %.4f | %.4f | %.0f | %.3f | %.1f |" % (
                    B, N, D, Q, m, nbytes / 1e9, nbytes / m / 1e6, nbytes / m / 1e6 / 8000.0, B * N / m / 1e6))
                sys.stdout.flush()
            del packed
            torch.cuda.empty_cache()
        return

    if args.scores:
        print("| batch x N x D | Q | kernel | mean ms | bytes moved (GB) | GB/s | of 8 TB/s | 2*Q*elements / time (Tflop/s) |")
        print("|---|---|---|---|---|---|---|---|")
        for (B, N, D) in [(256, 4096, 128), (2048, 4096, 128), (32, 131072, 128), (1, 1048576, 128), (4096, 4096, 64),
                          (512, 4096, 256), (1, 131072, 2048), (1, 131072, 4096), (1, 131072, 8192)]:
            E = B * N * D
            codes = torch.randint(-127, 128, (E,), dtype=torch.int8, device="cuda")
            scales = torch.rand(B * D, device="cuda") + 0.1
            for Q in (1, 2, 4, 8, 16):
                q = torch.randn(B * Q * D, device="cuda")
                out = torch.empty(B * Q * N, device="cuda")
                m, _ = timeit(lambda: kvq.kvq_scores_from_codes(q, Q, codes, scales, B, N, D, out))
                nbytes = E + 4.0 * B * Q * N + 4.0 * B * Q * D + 4.0 * B * D
                kind = "int8 MFMA" if (Q >= 3 and D % 64 == 0 and (D <= 1024 or (D % 256 == 0 and D <= 8192))) else "fp32 FMA"
                print("| %d x %d x %d | %d | %s | %.4f | %.4f | %.0f | %.3f | %.1f |" % (
                    B, N, D, Q, kind, m, nbytes / 1e9, nbytes / m / 1e6, nbytes / m / 1e6 / 8000.0, 2.0 * Q * E / m / 1e9))
                sys.stdout.flush()
            del codes
            torch.cuda.empty_cache()
        return

    if args.attn:
        print("| N x D | Q | form | (k, k_hat) ms | of 8 TB/s at 8 B/element | (k, codes) ms | of 8 TB/s at 5 B/element | fp32 matrix cores, (k, k_hat) ms |")
        print("|---|---|---|---|---|---|---|---|")
        mean = torch.zeros(1, dtype=torch.float64, device="cuda")
        saved = kvq.kvq_get_option(kvq.OPT_ATTN_FORM)
        for (N, D) in [(16384, 8192), (131072, 8192), (4096, 8192), (65536, 2048), (65536, 1024), (262144, 256),
                       (1048576, 128), (32768, 128), (16384, 8200)]:
            E = N * D
            x = torch.randn(E, device="cuda")
            scales = torch.empty(D, device="cuda")
            codes = torch.empty(E, dtype=torch.int8, device="cuda")
            xh = torch.empty(E, device="cuda")
            kvq.kvq_absmax_scales(x, scales, 1, N, D)
            kvq.kvq_quantize(x, scales, codes, 1, N, D)
            kvq.kvq_dequantize(codes, scales, xh, 1, N, D)
            for Q in (16, 64, 128):
                q = torch.randn(Q * D, device="cuda")
                kvq.kvq_set_option(kvq.OPT_ATTN_FORM, 0)
                m1, _ = timeit(lambda: kvq.kvq_attn_score_error(q, Q, x, xh, None, None, N, D, mean))
                m2, _ = timeit(lambda: kvq.kvq_attn_score_error(q, Q, x, None, codes, scales, N, D, mean))
                kvq.kvq_set_option(kvq.OPT_ATTN_FORM, 1)
                m3, _ = timeit(lambda: kvq.kvq_attn_score_error(q, Q, x, xh, None, None, N, D, mean))
                kvq.kvq_set_option(kvq.OPT_ATTN_FORM, saved)
                form = "bf16 pieces" if D % 128 == 0 else "fp32"
                print("| %d x %d | %d | %s | %.4f | %.3f | %.4f | %.3f | %.4f |" % (
                    N, D, Q, form, m1, 8.0 * E / m1 / 8e9, m2, 5.0 * E / m2 / 8e9, m3))
                sys.stdout.flush()
            del x, codes, xh
            torch.cuda.empty_cache()
        return

    if args.paper_sweep:
        names = [kvq.VARIANT_NAMES[v] for v in range(5)]
        print("| shape (T x D) | " + " | ".join("%s ms (GB/s)" % n for n in names) +
              " | dequantize ms (GB/s) | max-abs error | mean attention-score error (16 queries) |")
        print("|---|" + "---|" * (len(names) + 3))
        for label, (N, D) in W.PAPER_SHAPES.items():
            E = N * D
            x = torch.from_numpy(W.uniform_matrix(N, D, seed=0, stream=0)).cuda().reshape(-1)
            q = torch.from_numpy(W.uniform_matrix(16, D, seed=0, stream=1)).cuda()
            scales = torch.empty(D, dtype=torch.float32, device="cuda")
            codes = torch.empty(E, dtype=torch.int8, device="cuda")
            xh = torch.empty(E, dtype=torch.float32, device="cuda")
            ss = torch.zeros(1, dtype=torch.float64, device="cuda")
            mx = torch.zeros(1, dtype=torch.float32, device="cuda")
            mean = torch.zeros(1, dtype=torch.float64, device="cuda")
            kvq.kvq_absmax_scales(x, scales, 1, N, D)
            cells = []
            for v in range(5):
                m, _ = timeit(lambda: kvq.kvq_quantize_variant(v, x, scales, codes, 1, N, D))
                cells.append("%.4f (%.0f)" % (m, 5.0 * E / m / 1e6))
            m, _ = timeit(lambda: kvq.kvq_dequantize(codes, scales, xh, 1, N, D))
            cells.append("%.4f (%.0f)" % (m, 5.0 * E / m / 1e6))
            kvq.kvq_roundtrip_error(x, xh, None, None, 1, N, D, ss, mx)
            kvq.kvq_attn_score_error(q, 16, x, xh, None, None, N, D, mean)
            print("| %s (%d x %d) | %s | %.5f | %.4f |" % (label, N, D, " | ".join(cells), mx.item(), mean.item()))
            sys.stdout.flush()
            del x, codes, xh
            torch.cuda.empty_cache()
        return

    print("| cfg | shape | call | mean ms | min ms | algorithmic GB | GB/s (mean) | of 8 TB/s |")
    print("|---|---|---|---|---|---|---|---|")
    for cfg in [int(c) for c in args.configs.split(",")]:
        c = W.CONFIGS[cfg]
        x_np = W.generate(c)
        batch, N, D = c.batch, c.N, c.D
        E = c.elements
        x = torch.from_numpy(x_np.reshape(-1)).cuda()
        del x_np
        scales = torch.empty(batch * D, dtype=torch.float32, device="cuda")
        codes = torch.empty(E, dtype=torch.int8, device="cuda")
        xh = torch.empty(E, dtype=torch.float32, device="cuda")
        ss = torch.zeros(1, dtype=torch.float64, device="cuda")
        mx = torch.zeros(1, dtype=torch.float32, device="cuda")
        mean = torch.zeros(1, dtype=torch.float64, device="cuda")
        sb = 4.0 * batch * D
        calls = [
            ("absmax_scales", 4.0 * E + sb, lambda: kvq.kvq_absmax_scales(x, scales, batch, N, D)),
            ("quantize", 5.0 * E + sb, lambda: kvq.kvq_quantize(x, scales, codes, batch, N, D)),
            ("quantize_fused", 5.0 * E + sb, lambda: kvq.kvq_quantize_fused(x, scales, codes, batch, N, D)),
            ("dequantize", 5.0 * E + sb, lambda: kvq.kvq_dequantize(codes, scales, xh, batch, N, D)),
            ("roundtrip_error(x,x_hat)", 8.0 * E, lambda: kvq.kvq_roundtrip_error(x, xh, None, None, batch, N, D, ss, mx)),
            ("roundtrip_error(x,codes)", 5.0 * E + sb, lambda: kvq.kvq_roundtrip_error(x, None, codes, scales, batch, N, D, ss, mx)),
        ]
        if c.n_queries:
            Q = c.n_queries
            q = torch.from_numpy(W.queries(c)).cuda()
            calls.append(("attn_score_error(k,k_hat) Q=%d" % Q, 8.0 * E + 4.0 * Q * D,
                          lambda: kvq.kvq_attn_score_error(q, Q, x, xh, None, None, N, D, mean)))
            calls.append(("attn_score_error(k,codes) Q=%d" % Q, 5.0 * E + 4.0 * Q * D,
                          lambda: kvq.kvq_attn_score_error(q, Q, x, None, codes, scales, N, D, mean)))
        shape = "%dx%d" % (N, D) if batch == 1 else "%dx%dx%d" % (batch, N, D)
        for name, nbytes, f in calls:
            m, lo = timeit(f)
            gbps = nbytes / (m * 1e-3) / 1e9
            extra = ""
            if name.startswith("attn"):
                flops = 2.0 * c.n_queries * N * D
                if D % 128 == 0:   # the bf16 matrix-core form: six piece products per fp32 product
                    extra = " (%.0f TFLOP/s on the bf16 matrix cores, 6 piece products per product; bound: HBM, %.4f ms)" % (
                        6.0 * flops / (m * 1e-3) / 1e12, nbytes / 8e12 * 1e3)
                else:
                    bound_ms = max(flops / 157.3e12, nbytes / 8e12) * 1e3
                    extra = " (%.1f TFLOP/s on the fp32 matrix cores; %.2f of max(157.3 TFLOP/s, 8 TB/s) = %.4f ms)" % (
                        flops / (m * 1e-3) / 1e12, bound_ms / m, bound_ms)
            print("| %d | %s | %s | %.4f | %.4f | %.4f | %.0f%s | %.3f |" % (cfg, shape, name, m, lo, nbytes / 1e9, gbps, extra, gbps / 8000.0))
            sys.stdout.flush()
        del x, codes, xh
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
