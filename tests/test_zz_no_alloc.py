"""kvq_absmax_scales_static, the scale reduction for callers that cannot allocate device memory,
against kvq_absmax_scales (same kernels, the per-stream workspace) and against the CPU oracle:
bit-exact, on calls in a row that share the library's fixed scratch array, each smaller than the
one before, so that what an earlier call left in the array would show if a later one read it."""
import numpy as np
import pytest

import oracle
from paper_2601_04719_amd import kvq

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def both_ways(x_np):
    """(scales from the static entry point, scales from the allocating one), as numpy [batch, D]."""
    batch, N, D = x_np.shape
    x = torch.from_numpy(x_np).cuda()
    out = []
    for call in (kvq.kvq_absmax_scales_static, kvq.kvq_absmax_scales):
        s = torch.full((batch * D,), -3.0, dtype=torch.float32, device="cuda")
        call(x, s, batch, N, D)
        out.append(s.cpu().numpy().reshape(batch, D))
    return out


def matrix(rng, batch, N, D, spread):
    x = (rng.standard_normal((batch, N, D)) * np.exp(rng.uniform(-2, 2, (batch, 1, D))) * spread).astype(np.float32)
    x[:, :, D // 3] = 0.0
    x[0, N // 2, 0] = -1000.0 * spread       # absmax carried by one negative entry in the middle rows
    return x


def test_static_scale_reduction_two_calls_in_a_row_the_second_smaller():
    rng = np.random.default_rng(20260104)
    # the first call splits its rows over many chunks and fills a large part of the array with large maxima;
    # the later, smaller calls have values 1000x smaller, so a stale slot would win the maximum
    cases = [((1, 40000, 2048), 1000.0), ((1, 9000, 1024), 1.0), ((3, 700, 128), 1e-3), ((2, 33, 65), 1e-6)]
    for shape, spread in cases:
        x = matrix(rng, *shape, spread)
        s_static, s_alloc = both_ways(x)
        assert np.array_equal(bits(s_static), bits(s_alloc)), "static vs allocating entry point, %r" % (shape,)
        assert np.array_equal(bits(s_static), bits(oracle.compute_scales(x))), "static vs oracle, %r" % (shape,)
    # and the same first shape again after the small ones
    x = matrix(rng, *cases[0][0], 0.5)
    s_static, s_alloc = both_ways(x)
    assert np.array_equal(bits(s_static), bits(s_alloc))
    assert np.array_equal(bits(s_static), bits(oracle.compute_scales(x)))


def test_static_scale_reduction_rejects_what_its_scratch_cannot_hold():
    L = kvq.lib()
    fake = 0x1000    # never dereferenced: the size check comes before anything is enqueued
    D = kvq.STATIC_SCRATCH_FLOATS + 4
    assert L.kvq_absmax_scales_static(fake, fake, 1, 2, D, None) == kvq.ERR_LIMIT
    assert L.kvq_absmax_scales_static(fake, fake, D // 4, 2, 8, None) == kvq.ERR_LIMIT
    assert "KVQ_ERR_LIMIT" in kvq.kvq_status_string(kvq.ERR_LIMIT)
    with pytest.raises(kvq.KvqError) as e:
        kvq.kvq_absmax_scales_static(fake, fake, 1, 2, D)
    assert e.value.status == kvq.ERR_LIMIT
    # the largest channel count it takes: one row chunk per slab, still the same bits
    rng = np.random.default_rng(7)
    x = rng.standard_normal((1, 3, kvq.STATIC_SCRATCH_FLOATS)).astype(np.float32)
    s_static, s_alloc = both_ways(x)
    assert np.array_equal(bits(s_static), bits(s_alloc))
    assert np.array_equal(bits(s_static), bits(oracle.compute_scales(x)))
