"""Randomized parity sweep: seeded random shapes, misalignments and entry points against the oracle.

Complements the hand-picked shapes of test_gpu_parity.py; every case prints its parameters first so a
failure names itself.
"""
import numpy as np
import pytest

import oracle
import test_gpu_parity as T

pytestmark = pytest.mark.gpu

WIDTHS = [1, 2, 3, 4, 6, 8, 12, 16, 20, 31, 32, 48, 64, 66, 100, 128, 130, 192, 256, 320, 512, 1000, 1024, 1028, 2048,
          4096, 4100]


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_shapes_offsets_and_entry_points(seed):
    rng = np.random.default_rng(seed)
    for case in range(120):
        D = int(rng.choice(WIDTHS))
        batch = int(rng.choice([1, 1, 2, 3, 5]))
        N = int(rng.integers(1, max(2, 200000 // (D * batch))))
        off = int(rng.choice([0, 0, 0, 1, 2, 3, 4, 5, 8, 16]))
        kind = int(rng.integers(0, 6))
        tag = "seed %d case %d: kind %d shape (%d,%d,%d) offset %d" % (seed, case, kind, batch, N, D, off)
        print(tag, flush=True)
        x = T.make_matrix(rng, batch, N, D)
        if kind == 0:
            qs = rng.standard_normal((4, D)).astype(np.float32) if batch == 1 else None
            T.full_round_trip_check(x, qs, offset=off, tag=tag)
        elif kind == 1:
            if D % 2 == 0:
                T.int4_round_trip(x, offset=off)
        elif kind == 2:
            T.fp8_round_trip(x, offset=off)
        elif kind == 3:
            Q = int(rng.integers(1, 20))
            T.check_scores(x, rng.standard_normal((batch, Q, D)).astype(np.float32), Q, offset=off)
        elif kind == 4:
            cap = N + int(rng.integers(0, 5))
            g = T.GpuCache(batch, cap, D, off)
            ref_codes = np.full((batch, cap, D), 55, dtype=np.int8)
            ref_scales = np.zeros((batch, D), dtype=np.float32)
            xs = T.growing_tokens(rng, batch, N, D) if N > 1 else x
            done = 0
            while done < N:
                m = int(min(N - done, rng.choice([1, 1, 2, 7, 16, 17, 40, 300])))
                g.append(xs[:, done:done + m])
                ref_codes, ref_scales, _ = oracle.append(ref_codes, ref_scales, done, xs[:, done:done + m])
                done += m
            codes, scales, _ = g.state()
            T.assert_bits_equal(scales, ref_scales, tag + " scales")
            T.assert_bits_equal(codes, ref_codes, tag + " cache")
            assert g.guards_intact(), tag
        else:
            g = T.Gpu(x, offset=off)
            s_ref = oracle.compute_scales(x)
            sc, cd = g.quantize_fused()
            T.assert_bits_equal(sc, s_ref, tag + " fused scales")
            T.assert_bits_equal(cd, oracle.quantize(x, s_ref), tag + " fused codes")
            assert g.guards_intact(), tag


@pytest.mark.parametrize("seed", [30, 31])
def test_random_shapes_fused_call_on_tall_slabs(seed):
    """kvq_quantize_fused on slabs of 257 to 4096 rows, by the default choice of kernel and with the persistent
    one wherever its tiles are at least half full: any width that is a multiple of 4, few and many slabs
    (one tile or several per workgroup), buffers at and off 16-byte alignment (off it: two passes)."""
    from paper_2601_04719_amd import kvq
    rng = np.random.default_rng(seed)
    saved = kvq.kvq_get_option(kvq.OPT_FUSED_TALL)
    try:
        for case in range(24):
            N = int(rng.integers(2049, 4097)) if case % 3 == 0 else int(rng.integers(257, 2049))
            D = int(rng.choice([4, 8, 20, 32, 36, 64, 100, 128, 132, 256, 260, 516, 1024]))
            batch = int(rng.integers(1, max(2, min(400, 9000000 // (N * D)))))
            off = int(rng.choice([0, 0, 4, 8, 1, 2]))
            mode = 3 if case % 2 else 1
            tag = "seed %d case %d: shape (%d,%d,%d) offset %d mode %d" % (seed, case, batch, N, D, off, mode)
            print(tag, flush=True)
            kvq.kvq_set_option(kvq.OPT_FUSED_TALL, mode)
            x = T.make_matrix(rng, batch, N, D)
            g = T.Gpu(x, offset=off)
            s_ref = oracle.compute_scales(x)
            sc, cd = g.quantize_fused()
            T.assert_bits_equal(sc, s_ref, tag + " fused scales")
            T.assert_bits_equal(cd, oracle.quantize(x, s_ref), tag + " fused codes")
            assert g.guards_intact(), tag
    finally:
        kvq.kvq_set_option(kvq.OPT_FUSED_TALL, saved)


@pytest.mark.parametrize("seed", [10, 11])
def test_random_shapes_sixteen_bit_inputs_and_wide_rows(seed):
    """fp16 / bf16 matrices and appended tokens, and fp32 round trips on rows wide enough for the
    row-spanning reductions, with up to 3 M elements so that slabs split into many row chunks."""
    import torch
    from paper_2601_04719_amd import kvq
    rng = np.random.default_rng(seed)
    for case in range(70):
        kind = int(rng.integers(0, 3))
        D = int(rng.choice(WIDTHS if kind < 2 else [2048, 2052, 4096, 6144, 8192, 8200, 16384]))
        batch = int(rng.choice([1, 1, 2, 3]))
        N = int(rng.integers(1, max(2, int(rng.choice([200000, 3000000])) // (D * batch))))
        off = int(rng.choice([0, 0, 0, 1, 2, 4, 8, 16]))
        fmt = str(rng.choice(["f16", "bf16"]))
        dt = kvq.DTYPE_F16 if fmt == "f16" else kvq.DTYPE_BF16
        tag = "seed %d case %d: kind %d %s shape (%d,%d,%d) offset %d" % (seed, case, kind, fmt, batch, N, D, off)
        print(tag, flush=True)
        x = T.make_matrix(rng, batch, N, D)
        if kind == 0:
            x16 = oracle.narrow16(np.clip(x, -60000, 60000), fmt)
            xw = oracle.widen16(x16, fmt)
            s_ref = oracle.compute_scales(xw)
            q_ref = oracle.quantize(xw, s_ref)
            xh_ref = oracle.dequantize_as(q_ref, s_ref, fmt)
            n = x.size
            xd = torch.zeros(n + 16, dtype=torch.int16, device="cuda")
            xd[off:off + n].copy_(torch.from_numpy(x16.view(np.int16).reshape(-1)))
            scales = torch.full((batch * D + 16,), -5.0, dtype=torch.float32, device="cuda")
            codes = torch.full((n + 16,), 99, dtype=torch.int8, device="cuda")
            xh = torch.full((n + 16,), 12345, dtype=torch.int16, device="cuda")
            sv, cv, hv, xv = scales[off:], codes[off:], xh[off:], xd[off:]
            kvq.kvq_absmax_scales_t(dt, xv, sv, batch, N, D)
            kvq.kvq_quantize_t(dt, xv, sv, cv, batch, N, D)
            kvq.kvq_dequantize_t(dt, cv, sv, hv, batch, N, D)
            T.assert_bits_equal(sv[:batch * D].cpu().numpy().reshape(batch, D), s_ref, tag + " scales")
            T.assert_bits_equal(cv[:n].cpu().numpy().reshape(x.shape), q_ref, tag + " codes")
            assert np.array_equal(hv[:n].cpu().numpy().view(np.uint16).reshape(x.shape), xh_ref), tag + " x_hat"
            assert bool((codes[:off] == 99).all() and (codes[off + n:] == 99).all()), tag
            assert bool((xh[:off] == 12345).all() and (xh[off + n:] == 12345).all()), tag
            assert bool((scales[:off] == -5.0).all() and (scales[off + batch * D:] == -5.0).all()), tag
        elif kind == 1:
            cap = N + int(rng.integers(0, 5))
            g = T.GpuCache(batch, cap, D, off)
            ref_codes = np.full((batch, cap, D), 55, dtype=np.int8)
            ref_scales = np.zeros((batch, D), dtype=np.float32)
            xs = T.growing_tokens(rng, batch, N, D) if N > 1 else x
            x16 = oracle.narrow16(np.clip(xs, -60000, 60000), fmt)
            xw = oracle.widen16(x16, fmt)
            done = 0
            while done < N:
                m = int(min(N - done, rng.choice([1, 1, 2, 7, 16, 17, 40, 300, 5000])))
                tok = np.ascontiguousarray(x16[:, done:done + m])
                buf = torch.zeros(tok.size + 64, dtype=torch.int16, device="cuda")
                xv = buf[off:off + tok.size]
                xv.copy_(torch.from_numpy(tok.view(np.int16).reshape(-1)))
                kvq.kvq_append_t(dt, xv, g.scales, g.prev, g.codes, batch, done, m, cap, D)
                ref_codes, ref_scales, _ = oracle.append(ref_codes, ref_scales, done,
                                                         np.ascontiguousarray(xw[:, done:done + m]))
                done += m
            codes, scales, _ = g.state()
            T.assert_bits_equal(scales, ref_scales, tag + " scales")
            T.assert_bits_equal(codes, ref_codes, tag + " cache")
            assert g.guards_intact(), tag
        else:
            qs = rng.standard_normal((3, D)).astype(np.float32) if batch == 1 else None
            T.full_round_trip_check(x, qs, offset=off, tag=tag)


@pytest.mark.parametrize("seed", [20, 21])
def test_random_shapes_attention_score_error(seed):
    """Both forms of the score error on random (tokens, channels, queries, misalignment): rows that are a
    multiple of 128 channels on aligned buffers take the bf16 matrix-core kernels (one or two query tiles per
    workgroup, 32- or 64-token tiles, one to many tiles per workgroup), everything else the fp32 ones."""
    rng = np.random.default_rng(seed)
    for case in range(40):
        D = int(rng.choice([128, 128, 256, 384, 512, 640, 1024, 2048, 100, 130, 64]))
        Q = int(rng.choice([1, 2, 5, 16, 31, 32, 33, 64, 65, 100, 140]))
        N = int(rng.integers(1, max(2, min(40000, 300_000_000 // (D * Q)))))
        off = int(rng.choice([0, 0, 0, 4, 1, 8]))
        tag = "seed %d case %d: N %d D %d Q %d offset %d" % (seed, case, N, D, Q, off)
        print(tag, flush=True)
        x = T.make_matrix(rng, 1, N, D)
        qs = (rng.standard_normal((Q, D)) * np.exp(rng.uniform(-2, 2, (Q, 1)))).astype(np.float32)
        g = T.Gpu(x, offset=off)
        s_ref = oracle.compute_scales(x)
        q_ref = oracle.quantize(x, s_ref)
        xh_ref = oracle.dequantize(q_ref, s_ref)
        g.set_scales(s_ref)
        g.codes.copy_(T.torch.from_numpy(q_ref.reshape(-1)))
        g.xh.copy_(T.torch.from_numpy(xh_ref.reshape(-1)))
        a_ref = oracle.attn_score_error(qs, x[0], xh_ref[0])
        bound = T.attn_error_bound(qs, x[0], xh_ref[0])
        for from_codes in (False, True):
            a = g.attn_score_error(qs, from_codes)
            assert a == pytest.approx(a_ref, rel=T.REL, abs=0), tag + " from_codes=%s" % from_codes
            assert abs(a - a_ref) <= bound + 1e-13 * a_ref, tag + " beyond its rounding bound"
        assert g.guards_intact(), tag
