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
