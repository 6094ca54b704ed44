"""Times every entry point of libkvq.so on each of the five configurations and prints a markdown table.

Usage:  python -m paper_2601_04719_amd.report [--configs 1,2,3,4,5] [--iters 20]
Inputs are the seeded synthetic workloads, resident in HBM before timing; times are HIP-event
minima and means over `iters` launches on torch's current stream.
"""
import argparse
import sys

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="1,2,3,4,5")
    ap.add_argument("--iters", type=int, default=20)
    args = ap.parse_args()
    import torch
    from . import kvq, workloads as W

    stream = torch.cuda.current_stream()

    def timeit(f):
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.iters + 1)]
        ev[0].record(stream)
        for i in range(args.iters):
            f()
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        t = [ev[i].elapsed_time(ev[i + 1]) for i in range(args.iters)]
        return float(np.mean(t)), float(np.min(t))

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
                tf = 2.0 * c.n_queries * N * D / (m * 1e-3) / 1e12
                extra = " (%.1f TFLOP/s fp64, %.2f of 78.6)" % (tf, tf / 78.6)
            print("| %d | %s | %s | %.4f | %.4f | %.4f | %.0f%s | %.3f |" % (cfg, shape, name, m, lo, nbytes / 1e9, gbps, extra, gbps / 8000.0))
            sys.stdout.flush()
        del x, codes, xh
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
