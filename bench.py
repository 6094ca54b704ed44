#!/usr/bin/env python3
"""Benchmark of the INT8 KV-cache quantization hot path on one MI355X.

A step is one pass of the whole path over one resident batch:
    kvq_absmax_scales -> kvq_quantize -> kvq_dequantize -> kvq_roundtrip_error (x vs x_hat)
on the 1B-element stress configuration (fp32 [131072 x 8192], Student-t(3) entries times a
log-uniform per-channel spread, 1 % of channels all zero).  Inputs are generated on the host from a
fixed seed and copied to HBM before the timed region.

Prints one JSON line.  `value` is the headline metric of this workload, "quant+dequant GB/s": the
algorithmic bytes of quantize (4 B read + 1 B written per element) plus dequantize (1 B + 4 B)
divided by the summed mean durations of those two calls inside the timed steps, measured with HIP
events on the launch stream.  Every call's own time, GB/s and fraction of the 8 TB/s HBM peak are
under "kernels"; "roofline" repeats the entry of the call that takes the largest share of a step.

What the line says about itself: `traffic` values are HBM bytes per launch taken from the committed
rocprofv3 --pmc summary named in `traffic_source` (with the commit it was measured at), not counters
of this run; every timed call carries the shader clock measured while it ran (`sclk_GHz`: a one-
wavefront kernel on a second stream reads the shader-clock counter against the 100 MHz wall clock),
and rocm-smi's clock reading before and after the extra entry points is recorded as well.
"""
import argparse
import json
import os
import re
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=15)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--rows", type=int, default=0, help="use only the first ROWS tokens (debug)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip timing the entry points outside the step")
    ap.add_argument("--cpu-rows", type=int, default=0,
                    help="tokens of the workload the CPU oracle is timed on (0 = all of them, about a minute)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed steps, run one plain fp32 copy of the input (a dispatch of known "
                         "traffic, 4 B read + 4 B written per element) so that rocprofv3 --pmc counters can be scaled")
    ap.add_argument("--opt", action="append", default=[], metavar="KEY=VALUE",
                    help="library launch option, e.g. width=4 unroll=2 blocks_per_cu=8 nontemporal=1 block_threads=256 passes_per_block=1")
    return ap.parse_args()


def traffic_file(workload):
    return os.path.join("profiles", "hbm_traffic_%s.txt" % workload.split("[")[0])


def committed_traffic(kernel, workload):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, traffic_file(workload))
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"\s*traffic_bytes_per_launch\[(\w+)\]\s*=\s*([0-9.eE+]+)", line)
        if m and m.group(1) == kernel:
            return float(m.group(2))
    return None


def traffic_source(workload):
    """Where `traffic` comes from: the summary file and the commit its header says it was measured at."""
    path = os.path.join(ROOT, traffic_file(workload))
    if not os.path.exists(path):
        return None
    m = re.search(r"measured_at_commit\s*=\s*(\w+)", open(path).read())
    return {"file": traffic_file(workload), "measured_at_commit": m.group(1) if m else None,
            "kind": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command, scaled by a plain copy"}


def rocm_smi_sclk():
    """Shader clock in MHz as rocm-smi reports it right now, or None (the GPU is idle when this is called)."""
    try:
        p = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=20)
        data = json.loads(p.stdout)
        for card in data.values():
            for key, val in card.items():
                if key.lower().startswith("sclk"):
                    m = re.search(r"(\d+)\s*mhz", str(val).lower())
                    if m:
                        return int(m.group(1))
    except Exception:
        pass
    return None


class Timer:
    """Times one call at a time on the launch stream: its own warm-up (by time, so that clocks have settled
    for this kernel), then per-launch HIP events, then the shader clock while the same call keeps running."""

    def __init__(self, kvq, torch, stream):
        self.kvq, self.torch, self.stream = kvq, torch, stream
        self.side = torch.cuda.Stream()              # default priority, only ever runs the clock probe
        self.ticks = torch.zeros(2, dtype=torch.int64, device="cuda")

    def time(self, f, launches=10, warm_s=0.03):
        torch = self.torch
        t_end = time.perf_counter() + warm_s
        n = 0
        while n < 5 or time.perf_counter() < t_end:
            f()
            n += 1
            if n % 5 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(launches + 1)]
        ev[0].record(self.stream)
        for i in range(launches):
            f()
            ev[i + 1].record(self.stream)
        torch.cuda.synchronize()
        t = [ev[i].elapsed_time(ev[i + 1]) for i in range(launches)]
        return sum(t) / len(t), min(t)

    def sclk_during(self, f, mean_ms, window_us=3000):
        """Shader clock in GHz over a window in which f keeps the GPU busy, or None."""
        torch, kvq = self.torch, self.kvq
        try:
            calls = max(2, int(window_us * 1e-3 / max(mean_ms, 1e-3)) + 2)
            f()
            self.ticks.zero_()
            torch.cuda.synchronize()
            f()                                          # the GPU is busy when the probe starts
            kvq.kvq_probe_clock(self.ticks, window_us, stream=self.side.cuda_stream)
            for _ in range(calls):
                f()
            torch.cuda.synchronize()
            shader, wall = (int(v) for v in self.ticks.tolist())
            return round(0.1 * shader / wall, 3) if wall > 0 else None
        except Exception:
            return None


def time_extras(kvq, torch, timer, h, x, x_hat, codes, scales, E, N, D):
    """The entry points outside the timed step, on the workload's buffers: mean and min ms of 10 launches after
    each call's own warm-up, and the shader clock while it runs."""
    def row(f, nbytes=None, **more):
        mean, mn = timer.time(f)
        r = {"ms_mean": round(mean, 4), "ms_min": round(mn, 4)}
        if nbytes is not None:
            r["GBps"] = round(nbytes / (mean * 1e-3) / 1e9, 1)
            r["frac_hbm_peak"] = round(nbytes / (mean * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)
        r["sclk_GHz"] = timer.sclk_during(f, mean)
        r.update(more)
        return r

    out = {}
    saved = scales.clone()
    u8 = codes.view(torch.uint8)
    # the attention-score error of the step's own reconstruction (x_hat, codes and scales are as the step left
    # them), 64 queries: on the first 16384 tokens (the shape of configuration 4) and on all of them
    mean_abs = torch.zeros(1, dtype=torch.float64, device=x.device)
    q64 = torch.randn(64 * D, device=x.device)
    for rows in (min(16384, N), N):
        nb = 8.0 * rows * D + 4.0 * 64 * D
        out["attn_score_error_Q64[%dx%d]" % (rows, D)] = row(
            lambda: kvq.kvq_attn_score_error(q64, 64, x, x_hat, None, None, rows, D, mean_abs, stream=h), nb,
            note="k vs k_hat, 8 B per element; bf16 matrix cores")
        out["attn_score_error_from_codes_Q64[%dx%d]" % (rows, D)] = row(
            lambda: kvq.kvq_attn_score_error(q64, 64, x, None, codes, scales, rows, D, mean_abs, stream=h),
            5.0 * rows * D + 4.0 * 64 * D + 4.0 * D, note="k vs codes, 5 B per element")
    out["absmax_scales_fp8+quantize_fp8"] = row(lambda: (kvq.kvq_absmax_scales_fp8(x, scales, 1, N, D, stream=h),
                                                         kvq.kvq_quantize_fp8(x, scales, u8, 1, N, D, stream=h))[1],
                                                9.0 * E, note="two calls, 4 + 5 B per element")
    out["dequantize_fp8"] = row(lambda: kvq.kvq_dequantize_fp8(u8, scales, x_hat, 1, N, D, stream=h), 5.0 * E)
    kvq.kvq_absmax_scales_int4(x, scales, 1, N, D, stream=h)
    packed = u8[:E // 2]
    out["quantize_int4"] = row(lambda: kvq.kvq_quantize_int4(x, scales, packed, 1, N, D, stream=h), 4.5 * E)
    out["dequantize_int4"] = row(lambda: kvq.kvq_dequantize_int4(packed, scales, x_hat, 1, N, D, stream=h), 4.5 * E)
    # decode-like view of the same bytes: 2048-slab-per-GiB cache [B, 4096, 128]
    scales.copy_(saved)
    kvq.kvq_quantize(x, scales, codes, 1, N, D, stream=h)
    B = E // (4096 * 128)
    s2 = torch.rand(B * 128, device=x.device) + 0.5
    prev = torch.empty_like(s2)
    for Q in (1, 8):
        q = torch.randn(B * Q * 128, device=x.device)
        o = torch.empty(B * Q * 4096, device=x.device)
        nbytes = E + 4.0 * B * Q * 4096 + 4.0 * B * Q * 128 + 4.0 * B * 128
        out["scores_from_codes_Q%d" % Q] = row(lambda: kvq.kvq_scores_from_codes(q, Q, codes, s2, B, 4096, 128, o,
                                                                                 stream=h), nbytes)
    p4 = u8[:E // 2]                                    # any bytes are valid packed 4-bit codes
    for Q in (1, 8):
        q = torch.randn(B * Q * 128, device=x.device)
        o = torch.empty(B * Q * 4096, device=x.device)
        nbytes = E / 2 + 4.0 * B * Q * 4096 + 4.0 * B * Q * 128 + 4.0 * B * 128
        out["scores_from_codes_int4_Q%d" % Q] = row(lambda: kvq.kvq_scores_from_codes_int4(q, Q, p4, s2, B, 4096, 128,
                                                                                           o, stream=h), nbytes)
    tok = (torch.rand(B, 1, 128, device=x.device) - 0.5) * s2.view(B, 1, 128) * 100.0   # inside the range: no growth
    s3 = s2.clone()
    out["append_one_token_no_growth"] = row(lambda: kvq.kvq_append(tok, s3, prev, codes, B, 4095, 1, 4096, 128, stream=h),
                                            cache="[%d x 4096 x 128]" % B)
    tok16 = tok.to(torch.bfloat16)
    out["append_one_bf16_token_no_growth"] = row(lambda: kvq.kvq_append_t(kvq.DTYPE_BF16, tok16, s3, prev, codes, B, 4095,
                                                                          1, 4096, 128, stream=h),
                                                 cache="[%d x 4096 x 128]" % B)
    tok4 = tok * (7.0 / 127.0)                          # inside the 4-bit range of the same scales
    out["append_int4_one_token_no_growth"] = row(lambda: kvq.kvq_append_int4(tok4, s3, prev, p4, B // 2, 4095, 1, 4096,
                                                                             128, stream=h),
                                                 cache="[%d x 4096 x 128] 4-bit" % (B // 2))
    # scales and codes in one pass over x, on the decode-like view (a 32-channel column tile of a slab on chip)
    sf = torch.empty(B * 128, device=x.device)
    out["quantize_fused[%dx4096x128]" % B] = row(lambda: kvq.kvq_quantize_fused(x, sf, codes, B, 4096, 128, stream=h),
                                                 5.0 * E + 4.0 * B * 128, note="two calls move 9 B per element")
    # the workload as a bf16 matrix (2 B in, 1 B out per element)
    x16 = x.to(torch.bfloat16)
    kvq.kvq_absmax_scales_t(kvq.DTYPE_BF16, x16, scales, 1, N, D, stream=h)
    out["quantize_bf16"] = row(lambda: kvq.kvq_quantize_t(kvq.DTYPE_BF16, x16, scales, codes, 1, N, D, stream=h), 3.0 * E)
    out["dequantize_bf16"] = row(lambda: kvq.kvq_dequantize_t(kvq.DTYPE_BF16, codes, scales, x16, 1, N, D, stream=h),
                                 3.0 * E)
    del x16
    scales.copy_(saved)
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus %d refused)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU only: WORLD_SIZE must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2601_04719_amd import kvq, workloads as W

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    kvq.lib()   # fail loudly now if the HIP library is not built

    optkeys = {"width": kvq.OPT_CODEC_WIDTH, "unroll": kvq.OPT_CODEC_UNROLL,
               "blocks_per_cu": kvq.OPT_BLOCKS_PER_CU, "nontemporal": kvq.OPT_NONTEMPORAL,
               "block_threads": kvq.OPT_BLOCK_THREADS, "passes_per_block": kvq.OPT_PASSES_PER_BLOCK,
               "absmax_unroll": kvq.OPT_ABSMAX_UNROLL, "absmax_passes": kvq.OPT_ABSMAX_PASSES,
               "absmax_span": kvq.OPT_ABSMAX_SPAN, "absmax_blocks_per_cu": kvq.OPT_ABSMAX_BLOCKS_PER_CU}
    for kv in args.opt:
        k, v = kv.split("=")
        kvq.kvq_set_option(optkeys[k], int(v))
    opts = {k: kvq.kvq_get_option(v) for k, v in optkeys.items()}

    c = W.CONFIGS[args.config]
    N = args.rows if args.rows else c.N
    batch, D = c.batch, c.D
    E = batch * N * D
    t0 = time.time()
    x_host = W.generate(c, rows=(0, N))
    t_gen = time.time() - t0
    dev = torch.device("cuda:0")
    x = torch.empty(E, dtype=torch.float32, device=dev)
    x.copy_(torch.from_numpy(x_host.reshape(-1)))
    scales = torch.empty(batch * D, dtype=torch.float32, device=dev)
    codes = torch.empty(E, dtype=torch.int8, device=dev)
    x_hat = torch.empty(E, dtype=torch.float32, device=dev)
    sumsq = torch.zeros(1, dtype=torch.float64, device=dev)
    maxabs = torch.zeros(1, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    h = stream.cuda_stream
    names = ["absmax_scales", "quantize", "dequantize", "roundtrip_error"]
    alg_bytes = {"absmax_scales": 4.0 * E + 4.0 * batch * D,
                 "quantize": 5.0 * E + 4.0 * batch * D,
                 "dequantize": 5.0 * E + 4.0 * batch * D,
                 "roundtrip_error": 8.0 * E}

    def step(events=None):
        if events:
            events[0].record(stream)
        kvq.kvq_absmax_scales(x, scales, batch, N, D, stream=h)
        if events:
            events[1].record(stream)
        kvq.kvq_quantize(x, scales, codes, batch, N, D, stream=h)
        if events:
            events[2].record(stream)
        kvq.kvq_dequantize(codes, scales, x_hat, batch, N, D, stream=h)
        if events:
            events[3].record(stream)
        kvq.kvq_roundtrip_error(x, x_hat, None, None, batch, N, D, sumsq, maxabs, stream=h)
        if events:
            events[4].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(ev[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    if args.calibration_copy:
        x_hat.copy_(x)
        torch.cuda.synchronize()

    ms = {n: [ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(args.steps)] for j, n in enumerate(names)}
    mean_ms = {n: float(np.mean(v)) for n, v in ms.items()}
    kernels = {}
    for n in names:
        gbps = alg_bytes[n] / (mean_ms[n] * 1e-3) / 1e9
        kernels[n] = {"ms_mean": round(mean_ms[n], 4), "ms_min": round(float(np.min(ms[n])), 4),
                      "alg_GB": round(alg_bytes[n] / 1e9, 4), "GBps": round(gbps, 1),
                      "frac_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
                      "traffic": committed_traffic(n, c.name) if N == c.N else None}
    qd_bytes = alg_bytes["quantize"] + alg_bytes["dequantize"]
    qd_ms = mean_ms["quantize"] + mean_ms["dequantize"]
    value = qd_bytes / (qd_ms * 1e-3) / 1e9
    dominant = max(names, key=lambda n: mean_ms[n])
    workload = c.name if N == c.N else "%s first %d rows" % (c.name, N)
    # shader clock while each call of the step runs (after the timed region, one call at a time)
    timer = Timer(kvq, torch, stream)
    calls = {"absmax_scales": lambda: kvq.kvq_absmax_scales(x, scales, batch, N, D, stream=h),
             "quantize": lambda: kvq.kvq_quantize(x, scales, codes, batch, N, D, stream=h),
             "dequantize": lambda: kvq.kvq_dequantize(codes, scales, x_hat, batch, N, D, stream=h),
             "roundtrip_error": lambda: kvq.kvq_roundtrip_error(x, x_hat, None, None, batch, N, D, sumsq, maxabs,
                                                                stream=h)}
    for n in names:
        kernels[n]["sclk_GHz"] = timer.sclk_during(calls[n], mean_ms[n])
    roofline = {"kernel": "kvq_" + dominant, "bound": "hbm",
                "achieved": kernels[dominant]["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": kernels[dominant]["frac_hbm_peak"],
                "traffic": kernels[dominant]["traffic"],
                "traffic_source": traffic_source(c.name) if N == c.N else None}

    # sanity of what was timed: the run must have produced the statistics of a real round trip
    ss, mx = float(sumsq.item()), float(maxabs.item())
    s_max = float(scales.max().item())
    if not (ss > 0 and 0 < mx <= s_max / 2 * (1 + 2.0 ** -15)):
        print("round-trip statistics look wrong: sumsq=%r maxabs=%r max scale=%r" % (ss, mx, s_max), file=sys.stderr)
        sys.exit(1)

    # measured no-math streaming ceilings of this GPU for the same traffic patterns (context for `frac`)
    def probe(mode, nbytes):
        mean, _ = timer.time(lambda: kvq.kvq_probe_stream(mode, x, x_hat, codes, codes, scales, batch, N, D, stream=h))
        return round(nbytes / (mean * 1e-3) / 1e9, 1)
    ceilings = {"read_only": probe(0, 4.0 * E), "write_only": probe(1, 4.0 * E),
                "read4_write1": probe(2, 5.0 * E), "read1_write4": probe(3, 5.0 * E), "unit": "GB/s",
                "note": "kvq_probe_stream: flat one-shot read / write kernels, and the production quantize / "
                        "dequantize kernels with their arithmetic compiled out"}

    # the other entry points on the same buffers, outside the timed step: context, never part of `value`
    extras = None
    smi = None
    if not args.no_extras and N == c.N and batch == 1 and E % (4096 * 128) == 0:
        smi = {"before_extras": rocm_smi_sclk()}
        try:
            extras = time_extras(kvq, torch, timer, h, x, x_hat, codes, scales, E, N, D)
        except Exception as exc:  # a failure here must not cost the main line
            extras = {"error": repr(exc)}
        smi["after_extras"] = rocm_smi_sclk()
        smi["note"] = "rocm-smi between kernels (the GPU is idle at that moment); sclk_GHz of each call is measured while it runs"

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        # the oracle as it stands, one core, all four calls of the step; by default over the whole workload
        # (the column-outer scale computation of the paper's listing takes most of that time)
        rows = min(args.cpu_rows, N) if args.cpu_rows > 0 else N
        xs = x_host[0] if rows == N else np.ascontiguousarray(x_host[0, :rows])
        t = [time.perf_counter()]
        s_o = oracle.compute_scales(xs); t.append(time.perf_counter())
        q_o = oracle.quantize(xs, s_o); t.append(time.perf_counter())
        xh_o = oracle.dequantize(q_o, s_o); t.append(time.perf_counter())
        oracle.roundtrip_error(xs, xh_o); t.append(time.perf_counter())
        e = rows * D
        cpu_qd = (5.0 * e * 2) / (t[3] - t[1]) / 1e9
        cpu = {"value": round(cpu_qd, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": ("all %d tokens of %s" % (N, c.name) if rows == N else
                          "first %d of %d tokens of %s (slab 0)" % (rows, N, c.name)) +
                         "; quantize + dequantize, same byte count per element as `value`",
               "ms": {"absmax_scales": round((t[1] - t[0]) * 1e3, 1), "quantize": round((t[2] - t[1]) * 1e3, 1),
                      "dequantize": round((t[3] - t[2]) * 1e3, 1), "roundtrip_error": round((t[4] - t[3]) * 1e3, 1)},
               "step_GBps": round((4.0 + 5.0 + 5.0 + 8.0) * e / (t[4] - t[0]) / 1e9, 3),
               "host_cores_available": os.cpu_count()}
        del q_o, xh_o

    out = {
        "metric": "quant+dequant GB/s and % of HBM peak on 1B-element fp32 K (1 GPU)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload, "batch": batch, "N": N, "D": D, "elements": E, "seed": 0,
                   "step": "absmax_scales+quantize+dequantize+roundtrip_error(x,x_hat)", "options": opts},
        "frac_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        "step_GBps": round(sum(alg_bytes.values()) / (ms_per_step * 1e-3) / 1e9, 1),
        "kernels": kernels,
        "roofline": roofline,
        "measured_stream_ceilings": ceilings,
        "other_entry_points": extras,
        "rocm_smi_sclk_MHz": smi,
        "cpu_baseline": cpu,
        "result": {"l2_error": ss ** 0.5, "max_abs_error": mx},
        "host_generate_s": round(t_gen, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
