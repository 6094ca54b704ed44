"""Parity of the HIP library (through its C ABI) with the CPU oracle on the same seeded inputs.

Bars: scales, int8 codes and dequantized fp32 values bit-exact; error statistics within 1e-5
relative (both sides accumulate in fp64; only the summation order differs).
"""
import itertools
import zlib

import numpy as np
import pytest

import oracle
from paper_2601_04719_amd import kvq, workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

REL = 1e-5


def seed_of(*parts):
    """A seed that depends only on the case's parameters: the same in every process and on every
    Python build (the built-in hash of a str is salted per process)."""
    return zlib.crc32(repr(parts).encode())


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def assert_bits_equal(a, b, what):
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    assert a.shape == b.shape and a.dtype == b.dtype, what
    if a.dtype == np.float32:
        same = bits(a) == bits(b)
    else:
        same = a == b
    if not same.all():
        idx = np.argwhere(~same)[:5]
        raise AssertionError("%s: %d mismatches, first at %s: gpu %s oracle %s" % (
            what, (~same).sum(), idx.tolist(), [a[tuple(i)] for i in idx], [b[tuple(i)] for i in idx]))


def attn_error_bound(queries, k, k_hat):
    """Worst case of |gpu - exact| for kvq_attn_score_error.  The GPU forms e = k - k_hat exactly in fp32 and
    contracts it with the queries in runs of 64 channels whose results are added in fp64.  On the fp32 matrix
    cores a run is 64 products and 64 additions, each rounded once to fp32 (relative 2^-24): a score is off by
    at most 65 * 2^-24 * sum_d |q_d e_d|.  On the bf16 matrix cores e and q are each the exact sum of three bf16
    pieces and six of the nine piece products are kept: the dropped ones are below 2 * 2^-24 |q_d e_d| (+ 2^-32),
    the kept ones are exact in fp32, and the run is 24 matrix instructions on one fp32 accumulator, taken as
    at most two units in the last place each: (2 + 48) * 2^-24, inside the same 65 * 2^-24.  |.| and the mean
    are fp64 (negligible next to that).  The mean of |score| is then off by at most the mean of that bound.
    The errors are centred, so the observed difference is orders of magnitude smaller: the tests hold the
    call to the 1e-5 bar and to this bound."""
    e = np.abs(np.asarray(k, dtype=np.float64) - np.asarray(k_hat, dtype=np.float64))
    return 65 * 2.0 ** -24 * float((np.abs(np.asarray(queries, dtype=np.float64)) @ e.T).mean())


class Gpu:
    """Device buffers + calls through the binding for one [batch, N, D] problem."""

    def __init__(self, x_np, offset=0):
        x_np = np.ascontiguousarray(x_np, dtype=np.float32)
        if x_np.ndim == 2:
            x_np = x_np[None]
        self.shape = self.batch, self.N, self.D = x_np.shape
        self.offset = offset        # elements by which every buffer is shifted off its allocation
        n = x_np.size
        self._x = torch.empty(n + 64, dtype=torch.float32, device="cuda")
        self.x = self._x[offset:offset + n]
        self.x.copy_(torch.from_numpy(x_np.reshape(-1)))
        self._codes = torch.full((n + 64,), 99, dtype=torch.int8, device="cuda")
        self.codes = self._codes[offset:offset + n]
        self._xh = torch.full((n + 64,), 777.0, dtype=torch.float32, device="cuda")
        self.xh = self._xh[offset:offset + n]
        self._scales = torch.full((self.batch * self.D + 64,), -5.0, dtype=torch.float32, device="cuda")
        self.scales = self._scales[offset:offset + self.batch * self.D]
        self.sumsq = torch.zeros(1, dtype=torch.float64, device="cuda")
        self.maxabs = torch.zeros(1, dtype=torch.float32, device="cuda")
        self.mean = torch.zeros(1, dtype=torch.float64, device="cuda")

    def absmax_scales(self):
        kvq.kvq_absmax_scales(self.x, self.scales, self.batch, self.N, self.D)
        return self.scales.cpu().numpy().reshape(self.batch, self.D)

    def set_scales(self, s):
        self.scales.copy_(torch.from_numpy(np.ascontiguousarray(s, dtype=np.float32).reshape(-1)))

    def quantize(self):
        kvq.kvq_quantize(self.x, self.scales, self.codes, self.batch, self.N, self.D)
        return self.codes.cpu().numpy().reshape(self.shape)

    def quantize_fused(self):
        kvq.kvq_quantize_fused(self.x, self.scales, self.codes, self.batch, self.N, self.D)
        return (self.scales.cpu().numpy().reshape(self.batch, self.D),
                self.codes.cpu().numpy().reshape(self.shape))

    def dequantize(self):
        kvq.kvq_dequantize(self.codes, self.scales, self.xh, self.batch, self.N, self.D)
        return self.xh.cpu().numpy().reshape(self.shape)

    def roundtrip_error(self, from_codes):
        if from_codes:
            kvq.kvq_roundtrip_error(self.x, None, self.codes, self.scales, self.batch, self.N, self.D,
                                    self.sumsq, self.maxabs)
        else:
            kvq.kvq_roundtrip_error(self.x, self.xh, None, None, self.batch, self.N, self.D,
                                    self.sumsq, self.maxabs)
        return float(self.sumsq.item()), np.float32(self.maxabs.item())

    def attn_score_error(self, queries_np, from_codes):
        assert self.batch == 1
        q = torch.from_numpy(np.ascontiguousarray(queries_np, dtype=np.float32)).cuda()
        if from_codes:
            kvq.kvq_attn_score_error(q, q.shape[0], self.x, None, self.codes, self.scales, self.N, self.D,
                                     self.mean)
        else:
            kvq.kvq_attn_score_error(q, q.shape[0], self.x, self.xh, None, None, self.N, self.D, self.mean)
        return float(self.mean.item())

    def guards_intact(self):
        """Nothing was written outside [offset, offset+n) of any output buffer."""
        n = self.batch * self.N * self.D
        o = self.offset
        ok = bool((self._codes[:o] == 99).all() and (self._codes[o + n:] == 99).all())
        ok &= bool((self._xh[:o] == 777.0).all() and (self._xh[o + n:] == 777.0).all())
        ns = self.batch * self.D
        ok &= bool((self._scales[:o] == -5.0).all() and (self._scales[o + ns:] == -5.0).all())
        return ok


def full_round_trip_check(x_np, queries=None, offset=0, tag=""):
    """scales, codes, x_hat bit-exact; both forms of both error statistics within REL."""
    g = Gpu(x_np, offset=offset)
    x3 = x_np if x_np.ndim == 3 else x_np[None]
    s_ref = oracle.compute_scales(x3)
    assert_bits_equal(g.absmax_scales(), s_ref, tag + " scales")
    q_ref = oracle.quantize(x3, s_ref)
    assert_bits_equal(g.quantize(), q_ref, tag + " codes")
    xh_ref = oracle.dequantize(q_ref, s_ref)
    assert_bits_equal(g.dequantize(), xh_ref, tag + " x_hat")
    ss_ref, mx_ref = oracle.roundtrip_error(x3, xh_ref)
    for from_codes in (False, True):
        ss, mx = g.roundtrip_error(from_codes)
        assert ss == pytest.approx(ss_ref, rel=REL, abs=0), tag + " sumsq"
        assert mx == mx_ref, tag + " maxabs"
    if queries is not None:
        a_ref = oracle.attn_score_error(queries, x3[0], xh_ref[0])
        bound = attn_error_bound(queries, x3[0], xh_ref[0])
        for from_codes in (False, True):
            a = g.attn_score_error(queries, from_codes)
            assert a == pytest.approx(a_ref, rel=REL, abs=0), tag + " attn"
            assert abs(a - a_ref) <= bound + 1e-13 * a_ref, tag + " attn beyond its rounding bound"
    assert g.guards_intact(), tag + " wrote outside its buffers"
    # the one-call variant (single pass for small slabs, two passes otherwise) gives the same bits
    g2 = Gpu(x_np, offset=offset)
    s_f, q_f = g2.quantize_fused()
    assert_bits_equal(s_f, s_ref, tag + " fused scales")
    assert_bits_equal(q_f, q_ref, tag + " fused codes")
    assert g2.guards_intact(), tag + " fused wrote outside its buffers"
    return g


# ------------------------------------------------------------------ the five configurations
def test_config1_full():
    full_round_trip_check(W.generate(1)[0], W.queries(1), tag="cfg1")


def test_config2_full():
    full_round_trip_check(W.generate(2)[0], W.queries(2), tag="cfg2")


@pytest.mark.parametrize("tensor", [0, 1])
def test_config3_full_batched_k_and_v(tensor):
    x = W.generate(3, tensor=tensor)
    g = Gpu(x)
    s_ref = oracle.compute_scales(x)
    assert s_ref.shape == (256, 128)
    assert_bits_equal(g.absmax_scales(), s_ref, "cfg3 scales")
    q_ref = oracle.quantize(x, s_ref)
    assert_bits_equal(g.quantize(), q_ref, "cfg3 codes")
    xh_ref = oracle.dequantize(q_ref, s_ref)
    assert_bits_equal(g.dequantize(), xh_ref, "cfg3 x_hat")
    ss_ref, mx_ref = oracle.roundtrip_error(x, xh_ref)
    for from_codes in (False, True):
        ss, mx = g.roundtrip_error(from_codes)
        assert ss == pytest.approx(ss_ref, rel=REL, abs=0) and mx == mx_ref
    # the one-call variant gives the same bits
    g2 = Gpu(x)
    s_f, q_f = g2.quantize_fused()
    assert_bits_equal(s_f, s_ref, "cfg3 fused scales")
    assert_bits_equal(q_f, q_ref, "cfg3 fused codes")


def test_config4_full():
    x = W.generate(4)[0]
    g = Gpu(x)
    s_ref = oracle.compute_scales(x)
    assert_bits_equal(g.absmax_scales()[0], s_ref, "cfg4 scales")
    q_ref = oracle.quantize(x, s_ref)
    assert_bits_equal(g.quantize()[0], q_ref, "cfg4 codes")
    xh_ref = oracle.dequantize(q_ref, s_ref)
    assert_bits_equal(g.dequantize()[0], xh_ref, "cfg4 x_hat")
    # attention-score error (Evaluation, "Attention Score Error"): all 64 queries over all 16384 tokens on
    # both sides, both forms of the call
    qs = W.queries(4)
    a_ref = oracle.attn_score_error(qs, x, xh_ref)
    bound = attn_error_bound(qs, x, xh_ref)
    for from_codes in (False, True):
        a = g.attn_score_error(qs, from_codes)
        assert a == pytest.approx(a_ref, rel=REL, abs=0), "cfg4 attn (from_codes=%s)" % from_codes
        assert abs(a - a_ref) <= bound, "cfg4 attn beyond its rounding bound"
        assert abs(a - a_ref) <= 1e-7 * a_ref       # what centred rounding errors leave of it


def test_config5_full_size_against_oracle_in_row_chunks():
    c = W.CONFIGS[5]
    x = W.generate(5)[0]
    g = Gpu(x)
    s_ref = oracle.compute_scales(x)
    assert np.count_nonzero(s_ref == 0) == 82
    assert_bits_equal(g.absmax_scales()[0], s_ref, "cfg5 scales")
    g.quantize()
    g.dequantize()
    ss_gpu, mx_gpu = g.roundtrip_error(from_codes=False)
    ss_gpu2, mx_gpu2 = g.roundtrip_error(from_codes=True)
    ss_ref, mx_ref = 0.0, np.float32(0)
    rows = 8192
    for r0 in range(0, c.N, rows):
        xs = x[r0:r0 + rows]
        q_ref = oracle.quantize(xs, s_ref)
        q_gpu = g.codes[r0 * c.D:(r0 + rows) * c.D].cpu().numpy().reshape(rows, c.D)
        assert_bits_equal(q_gpu, q_ref, "cfg5 codes rows %d.." % r0)
        xh_ref = oracle.dequantize(q_ref, s_ref)
        xh_gpu = g.xh[r0 * c.D:(r0 + rows) * c.D].cpu().numpy().reshape(rows, c.D)
        assert_bits_equal(xh_gpu, xh_ref, "cfg5 x_hat rows %d.." % r0)
        ss, mx = oracle.roundtrip_error(xs, xh_ref)
        ss_ref += ss
        mx_ref = max(mx_ref, mx)
    assert ss_gpu == pytest.approx(ss_ref, rel=REL, abs=0) and mx_gpu == mx_ref
    assert ss_gpu2 == pytest.approx(ss_ref, rel=REL, abs=0) and mx_gpu2 == mx_ref


# ------------------------------------------------------------------ more work items than partial-result slots
# The error reductions keep one partial result per workgroup in 8192 slots; beyond that a workgroup
# takes several work items in turn.  These shapes have more items than slots in each such kernel.
@pytest.mark.parametrize("shape", [(9000, 8, 128), (9000, 1, 2048), (8200, 3, 4100)],
                         ids=lambda s: "x".join(map(str, s)))
def test_roundtrip_error_from_codes_with_more_slabs_than_partial_slots(shape):
    rng = np.random.default_rng(seed_of("many slabs", shape))
    x = make_matrix(rng, *shape)
    g = Gpu(x)
    s_ref = oracle.compute_scales(x)
    q_ref = oracle.quantize(x, s_ref)
    xh_ref = oracle.dequantize(q_ref, s_ref)
    g.set_scales(s_ref)
    g.codes.copy_(torch.from_numpy(q_ref.reshape(-1)))
    g.xh.copy_(torch.from_numpy(xh_ref.reshape(-1)))
    ss_ref, mx_ref = oracle.roundtrip_error(x, xh_ref)
    for from_codes in (True, False):
        ss, mx = g.roundtrip_error(from_codes)
        assert ss == pytest.approx(ss_ref, rel=REL, abs=0) and mx == mx_ref, "from_codes=%s" % from_codes
    # one slab's contribution must really be in the sum: perturb the last slab only
    g.x[-shape[1] * shape[2]:] += 1.0
    x[-1] += np.float32(1.0)
    ss_ref2, mx_ref2 = oracle.roundtrip_error(x, xh_ref)
    assert ss_ref2 > 1.5 * ss_ref
    for from_codes in (True, False):
        ss, mx = g.roundtrip_error(from_codes)
        assert ss == pytest.approx(ss_ref2, rel=REL, abs=0) and mx == mx_ref2, "last slab, from_codes=%s" % from_codes


@pytest.mark.parametrize("N,D,Q", [(600000, 8, 3), (530000, 5, 33)], ids=lambda v: str(v))
def test_attn_score_error_with_more_token_tiles_than_partial_slots(N, D, Q):
    rng = np.random.default_rng(seed_of("many tiles", N, D, Q))
    x = make_matrix(rng, 1, N, D)
    qs = rng.standard_normal((Q, D)).astype(np.float32)
    g = Gpu(x)
    s_ref = oracle.compute_scales(x)
    q_ref = oracle.quantize(x, s_ref)
    xh_ref = oracle.dequantize(q_ref, s_ref)
    g.set_scales(s_ref)
    g.codes.copy_(torch.from_numpy(q_ref.reshape(-1)))
    g.xh.copy_(torch.from_numpy(xh_ref.reshape(-1)))
    a_ref = oracle.attn_score_error(qs, x[0], xh_ref[0])
    for from_codes in (False, True):
        assert g.attn_score_error(qs, from_codes) == pytest.approx(a_ref, rel=REL, abs=0), "from_codes=%s" % from_codes
    # the last tokens must really be in the mean: move the reconstruction of the last 40 tokens only
    g.xh[-40 * D:] += 0.5
    xh_ref[0, -40:] += np.float32(0.5)
    a_ref2 = oracle.attn_score_error(qs, x[0], xh_ref[0])
    assert a_ref2 > a_ref * (1 + 1e-3)
    assert g.attn_score_error(qs, from_codes=False) == pytest.approx(a_ref2, rel=REL, abs=0)


# Shapes that take the bf16 matrix-core form (D a multiple of 128): a single ragged tile; 3 chunks; more tiles
# than compute units, so that workgroups walk several tiles, with one-chunk tiles (the hand-over area alternates),
# three query chunks, and 64-token tiles (N >= 64 tokens per compute unit) ending in a ragged one; few tiles.
@pytest.mark.parametrize("N,D,Q", [(1, 128, 1), (33, 128, 3), (100, 384, 33), (257, 256, 65), (9000, 128, 64),
                                   (5000, 640, 130), (40000, 128, 20), (16500, 256, 64), (33000, 128, 40),
                                   (70, 1024, 64)], ids=lambda v: str(v))
def test_attn_score_error_on_the_bf16_matrix_cores(N, D, Q):
    rng = np.random.default_rng(seed_of("bf16 pieces", N, D, Q))
    x = make_matrix(rng, 1, N, D)
    qs = (rng.standard_normal((Q, D)) * np.exp(rng.uniform(-3, 3, (Q, 1)))).astype(np.float32)
    g = Gpu(x)
    s_ref = oracle.compute_scales(x)
    q_ref = oracle.quantize(x, s_ref)
    xh_ref = oracle.dequantize(q_ref, s_ref)
    g.set_scales(s_ref)
    g.codes.copy_(torch.from_numpy(q_ref.reshape(-1)))
    g.xh.copy_(torch.from_numpy(xh_ref.reshape(-1)))
    a_ref = oracle.attn_score_error(qs, x[0], xh_ref[0])
    bound = attn_error_bound(qs, x[0], xh_ref[0])
    saved = kvq.kvq_get_option(kvq.OPT_ATTN_FORM)
    try:
        got = {}
        for form in (0, 1):            # 0: bf16 pieces (these shapes allow it), 1: fp32 matrix cores
            kvq.kvq_set_option(kvq.OPT_ATTN_FORM, form)
            for from_codes in (False, True):
                a = g.attn_score_error(qs, from_codes)
                assert a == pytest.approx(a_ref, rel=REL, abs=0), "form %d from_codes=%s" % (form, from_codes)
                assert abs(a - a_ref) <= bound + 1e-13 * a_ref, "form %d beyond its rounding bound" % form
                got[form, from_codes] = a
            assert got[form, False] == got[form, True]      # the same e either way, the same arithmetic
        kvq.kvq_set_option(kvq.OPT_ATTN_FORM, 0)
        assert g.attn_score_error(qs, False) == got[0, False]   # same bits run to run
        # the last tokens must really be in the mean: move the reconstruction of the last 3 tokens only
        m = min(3, N)
        g.xh[-m * D:] += 0.5
        xh_ref[0, -m:] += np.float32(0.5)
        a_ref2 = oracle.attn_score_error(qs, x[0], xh_ref[0])
        assert a_ref2 > a_ref
        assert g.attn_score_error(qs, from_codes=False) == pytest.approx(a_ref2, rel=REL, abs=0)
    finally:
        kvq.kvq_set_option(kvq.OPT_ATTN_FORM, saved)


def test_attn_score_error_single_scores_stay_within_the_rounding_bound():
    """One token and one query make the mean a single |score|, so the per-score bound can be held against the
    hardware directly: 300 random rows of 128-2048 channels with magnitudes spread over 2^-20 .. 2^20, all
    products of one sign (nothing cancels: the sum of magnitudes is the score) or of random sign, on the bf16
    matrix cores and on the fp32 ones.  The bound allows two units in the last place per 16-product matrix
    instruction; what is observed is printed."""
    rng = np.random.default_rng(seed_of("single scores"))
    saved = kvq.kvq_get_option(kvq.OPT_ATTN_FORM)
    worst = {0: 0.0, 1: 0.0}
    try:
        for case in range(300):
            D = int(rng.choice([128, 256, 512, 1024, 2048]))
            k = (rng.standard_normal((1, D)) * np.exp2(rng.uniform(-20, 20, (1, D)))).astype(np.float32)
            # a reconstruction a little off, as after quantization: k_hat = k (1 + up to 2^-8), rounded to fp32
            kh = (k.astype(np.float64) * (1.0 + rng.uniform(-1, 1, (1, D)) * 2.0 ** -8)).astype(np.float32)
            e = k.astype(np.float64) - kh.astype(np.float64)        # exact: k_hat is within a factor of two of k
            q = (rng.standard_normal((1, D)) * np.exp2(rng.uniform(-10, 10, (1, D)))).astype(np.float32)
            if case % 2 == 0:
                q = (np.abs(q) * np.where(e[0] < 0, -1.0, 1.0)).astype(np.float32)   # every product >= 0
            exact = abs(float((q.astype(np.float64) * e).sum()))
            mags = float(np.abs(q.astype(np.float64) * e).sum())
            g = Gpu(k)
            g.xh.copy_(torch.from_numpy(kh.reshape(-1)))
            for form in (0, 1):
                kvq.kvq_set_option(kvq.OPT_ATTN_FORM, form)
                got = g.attn_score_error(q, from_codes=False)
                err = abs(got - exact)
                assert err <= 65 * 2.0 ** -24 * mags, "case %d D %d form %d: off by %.3g of the sum of magnitudes" % (
                    case, D, form, err / mags)
                worst[form] = max(worst[form], err / mags)
    finally:
        kvq.kvq_set_option(kvq.OPT_ATTN_FORM, saved)
    print("largest |gpu - exact| / sum of magnitudes: bf16 form %.2f x 2^-24, fp32 form %.2f x 2^-24"
          % (worst[0] * 2.0 ** 24, worst[1] * 2.0 ** 24))


# ------------------------------------------------------------------ shapes, tails, alignment
def make_matrix(rng, batch, N, D):
    x = (rng.standard_normal((batch, N, D)) * np.exp(rng.uniform(-2, 2, (batch, 1, D)))).astype(np.float32)
    if D >= 3:
        x[:, :, 1] = 0.0                                   # an all-zero channel inside a nonzero matrix
        x[0, :, 2] = -np.abs(x[0, :, 2])                   # absmax carried by a negative entry
    if D >= 5 and N >= 4:
        s = np.float32(0.0625)                             # exact ties: multiples of s/2 with absmax 127 s
        x[:, :, 4] = (rng.integers(-253, 254, (batch, N)) * (s / 2)).astype(np.float32)
        x[:, 0, 4] = 127 * s
    if N >= 2:
        x[0, 1, 0] = -0.0
    return x


SHAPES = [(1, 1, 1), (1, 1, 3), (1, 2, 4), (1, 63, 5), (1, 64, 15), (1, 65, 16), (3, 5, 17), (1, 100, 63),
          (2, 33, 65), (1, 7, 100), (1, 300, 128), (2, 257, 1000), (1, 19, 4096), (1, 3, 4100), (1, 1000, 48),
          (5, 1, 272), (1, 2050, 8)]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_ragged_shapes(shape):
    rng = np.random.default_rng(seed_of(shape))
    x = make_matrix(rng, *shape)
    qs = rng.standard_normal((5, shape[2])).astype(np.float32) if shape[0] == 1 else None
    full_round_trip_check(x, qs, tag="shape %r" % (shape,))


@pytest.mark.parametrize("offset", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("shape", [(1, 70, 64), (2, 9, 256), (1, 130, 20)], ids=lambda s: "x".join(map(str, s)))
def test_unaligned_base_pointers(shape, offset):
    rng = np.random.default_rng(offset * 1000 + shape[1])
    x = make_matrix(rng, *shape)
    qs = rng.standard_normal((3, shape[2])).astype(np.float32) if shape[0] == 1 else None
    full_round_trip_check(x, qs, offset=offset, tag="offset %d" % offset)


# ------------------------------------------------------------------ the paper's four designs
@pytest.mark.parametrize("shape", [(1, 1, 1), (1, 5, 3), (2, 33, 65), (1, 300, 128), (3, 257, 1000), (1, 19, 4096),
                                   (1, 70, 20), (2, 1030, 256)], ids=lambda s: "x".join(map(str, s)))
def test_paper_kernel_designs_give_identical_codes(shape):
    """Cross-kernel consistency, as in the paper's unit tests: naive, tiled, coarsened, vectorized and the
    production kernel all agree with the oracle bit for bit (the paper allows +-1)."""
    rng = np.random.default_rng(sum(shape) + 7)
    x = make_matrix(rng, *shape)
    s_ref = oracle.compute_scales(x)
    q_ref = oracle.quantize(x, s_ref)
    g = Gpu(x)
    g.set_scales(s_ref)
    for variant, name in kvq.VARIANT_NAMES.items():
        g.codes.fill_(99)
        if variant == kvq.VARIANT_VECTORIZED and shape[2] % 4:
            with pytest.raises(kvq.KvqError) as e:
                kvq.kvq_quantize_variant(variant, g.x, g.scales, g.codes, *shape)
            assert e.value.status == kvq.ERR_ARG
            continue
        kvq.kvq_quantize_variant(variant, g.x, g.scales, g.codes, *shape)
        assert_bits_equal(g.codes.cpu().numpy().reshape(shape), q_ref, "%s codes" % name)
        assert g.guards_intact(), name
    with pytest.raises(kvq.KvqError):
        kvq.kvq_quantize_variant(9, g.x, g.scales, g.codes, *shape)


def test_paper_error_figures_on_the_gpu_path():
    """Inputs filled uniformly in [-1, 1], as in the paper's error experiment: the GPU path reproduces the
    printed max-abs error 0.00394 and the mean attention-score error 0.095 at D = 8192, and agrees with the
    oracle on the same inputs."""
    k = W.uniform_matrix(2048, 8192, seed=5, stream=0)
    qs = W.uniform_matrix(16, 8192, seed=5, stream=1)
    g = Gpu(k)
    s_ref = oracle.compute_scales(k)
    assert_bits_equal(g.absmax_scales()[0], s_ref, "scales")
    q_ref = oracle.quantize(k, s_ref)
    assert_bits_equal(g.quantize()[0], q_ref, "codes")
    kh_ref = oracle.dequantize(q_ref, s_ref)
    assert_bits_equal(g.dequantize()[0], kh_ref, "k_hat")
    ss_ref, mx_ref = oracle.roundtrip_error(k, kh_ref)
    ss, mx = g.roundtrip_error(from_codes=False)
    assert mx == mx_ref and ss == pytest.approx(ss_ref, rel=REL)
    assert abs(float(mx) - 0.00394) < 5e-6                       # Evaluation, "Reconstruction Error"
    a = g.attn_score_error(qs, from_codes=False)
    assert a == pytest.approx(oracle.attn_score_error(qs, k, kh_ref), rel=REL)
    assert abs(a - 0.095) < 0.0025                                # Evaluation, "Attention Score Error"


# ------------------------------------------------------------------ scores straight from the quantized cache
def scores_bound(D, fast):
    """Worst-case |gpu - exact| per unit of sum_d |q k_hat|: fp32 rounding of q*s (vs the oracle's
    rounding of code*s), one fp32 FMA per code in a lane's chain (16 per 1024-channel chunk, or D in
    the generic kernel), up to 6 cross-lane adds, and the final value kept in fp32."""
    n = 16 * -(-D // 1024) + 12 if fast else D + 4
    return n * 2.0 ** -24


def check_scores(x, qs, Q, offset=0):
    """kvq_scores_from_codes against the oracle, with the bound of the kernel the shape selects."""
    batch, N, D = x.shape
    s_ref = oracle.compute_scales(x)
    q_ref = oracle.quantize(x, s_ref)
    g = Gpu(x, offset=offset)
    g.set_scales(s_ref)
    g.codes.copy_(torch.from_numpy(q_ref.reshape(-1)))
    qd = torch.from_numpy(qs).cuda()
    out = torch.full((batch * Q * N + 8,), 555.0, dtype=torch.float32, device="cuda")
    kvq.kvq_scores_from_codes(qd, Q, g.codes, g.scales, batch, N, D, out)
    got = out[:batch * Q * N].cpu().numpy().reshape(batch, Q, N).astype(np.float64)
    assert bool((out[batch * Q * N:] == 555.0).all())
    matrix_cores = Q >= 3 and D % 64 == 0 and (D <= 1024 or (D % 256 == 0 and D <= 8192)) and offset % 16 == 0
    fast = D % 16 == 0 and offset % 16 == 0
    worst = 0.0
    for b in range(batch):
        ref = oracle.scores_from_codes(qs[b], q_ref[b], s_ref[b])
        xh = oracle.dequantize(q_ref[b], s_ref[b]).astype(np.float64)
        mag = np.abs(qs[b].astype(np.float64)) @ np.abs(xh).T                       # [Q, N]
        if matrix_cores:
            # 28-bit fixed point relative to each query's largest |q*s|; exact integer sums; one rounding
            top = np.abs(qs[b].astype(np.float64) * s_ref[b].astype(np.float64)).max(axis=1) * (1 + 2.0 ** -23)
            bound = 2.0 ** -27 * top[:, None] * np.abs(q_ref[b].astype(np.float64)).sum(axis=1)[None, :] \
                + 4 * 2.0 ** -24 * mag
        else:
            bound = scores_bound(D, fast) * mag
        # gradual underflow: a folded query q*s below 2^-126 carries an absolute error of up to 2^-150
        # per channel (times |code| <= 127), and so does the final rounding of the score
        bound = bound + (127 * D + 1) * 2.0 ** -150
        err = np.abs(got[b] - ref)
        assert (err <= bound).all(), (b, float((err / bound).max()))
        worst = max(worst, float((err / (mag + 1e-300)).max()))
    return worst


@pytest.mark.parametrize("shape,Q", [((1, 1024, 64), 16), ((1, 4096, 128), 1), ((6, 1000, 128), 8), ((3, 257, 128), 5),
                                     ((1, 300, 80), 3), ((2, 100, 1024), 2), ((1, 50, 4096), 9), ((1, 33, 100), 4),
                                     ((2, 1, 16), 1), ((1, 70, 20), 2), ((2, 700, 256), 4), ((1, 300, 2048), 3), ((1, 300, 1024), 3), ((2, 64, 192), 8),
                                     ((4, 33, 64), 7), ((1, 5000, 128), 13), ((3, 1, 128), 8),
                                     # rows of 1280-8192 channels: 16 / 8 / 4 queries per pass, whole and partial groups
                                     ((1, 300, 2048), 16), ((2, 77, 2048), 11), ((1, 40, 4096), 6), ((1, 33, 8192), 7),
                                     ((1, 100, 1280), 13), ((1, 2100, 4096), 8)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else "Q%d" % v)
def test_scores_from_codes(shape, Q):
    batch, N, D = shape
    rng = np.random.default_rng(N + D + Q)
    x = make_matrix(rng, batch, N, D)
    qs = rng.standard_normal((batch, Q, D)).astype(np.float32)
    check_scores(x, qs, Q)


def test_scores_from_codes_matrix_core_path_corner_cases():
    rng = np.random.default_rng(77)
    # outlier channels (x20) and the full code range: config 2
    x = W.generate(2)
    worst = check_scores(x, rng.standard_normal((1, 8, 128)).astype(np.float32), 8)
    assert worst < 2.0 ** -20
    # queries of very different magnitude, a zero query, tiny and huge values
    x = make_matrix(rng, 2, 200, 128)
    qs = rng.standard_normal((2, 6, 128)).astype(np.float32)
    qs[:, 1] *= 1e-30
    qs[:, 2] *= 1e30
    qs[:, 3] = 0.0
    qs[:, 4, :64] *= 1e-6
    check_scores(x, qs, 6)
    check_scores((x * np.float32(1e-36)).astype(np.float32), qs[:, :5], 5)
    # codes that are not 16-byte aligned take the vector path
    check_scores(x, qs, 6, offset=4)


# ------------------------------------------------------------------ fp16 / bf16 matrices
@pytest.mark.parametrize("fmt", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [(1, 1024, 64), (1, 4096, 128), (6, 1000, 128), (2, 257, 1000), (1, 19, 4096),
                                   (1, 300, 8192), (3, 5, 17), (1, 100, 63), (1, 1, 1), (1, 70, 20), (2, 2050, 8)],
                         ids=lambda s: "x".join(map(str, s)))
def test_sixteen_bit_matrices(shape, fmt):
    """Scales and codes of an fp16 / bf16 matrix equal those of the widened matrix (oracle); dequantization
    into the 16-bit format is the fp32 product rounded once, to nearest even.  All bit-exact."""
    rng = np.random.default_rng(sum(shape) + len(fmt))
    x32 = make_matrix(rng, *shape)
    if fmt == "f16":
        x32 = np.clip(x32, -60000, 60000)
    x16 = oracle.narrow16(x32, fmt)
    xw = oracle.widen16(x16, fmt)
    s_ref = oracle.compute_scales(xw)
    q_ref = oracle.quantize(xw, s_ref)
    xh_ref = oracle.dequantize_as(q_ref, s_ref, fmt)
    dt = kvq.DTYPE_F16 if fmt == "f16" else kvq.DTYPE_BF16
    batch, N, D = shape
    n = batch * N * D
    for offset in (0, 1):     # aligned, and shifted by one element (generic kernels)
        xd = torch.zeros(n + 16, dtype=torch.int16, device="cuda")
        xd[offset:offset + n].copy_(torch.from_numpy(x16.view(np.int16).reshape(-1)))
        scales = torch.full((batch * D + 16,), -5.0, dtype=torch.float32, device="cuda")
        codes = torch.full((n + 16,), 99, dtype=torch.int8, device="cuda")
        xh = torch.full((n + 16,), 12345, dtype=torch.int16, device="cuda")
        sv, cv, hv, xv = scales[offset:], codes[offset:], xh[offset:], xd[offset:]
        kvq.kvq_absmax_scales_t(dt, xv, sv, batch, N, D)
        kvq.kvq_quantize_t(dt, xv, sv, cv, batch, N, D)
        kvq.kvq_dequantize_t(dt, cv, sv, hv, batch, N, D)
        assert_bits_equal(sv[:batch * D].cpu().numpy().reshape(batch, D), s_ref, "%s scales" % fmt)
        assert_bits_equal(cv[:n].cpu().numpy().reshape(shape), q_ref, "%s codes" % fmt)
        got = hv[:n].cpu().numpy().view(np.uint16).reshape(shape)
        assert np.array_equal(got, xh_ref), "%s x_hat" % fmt
        assert bool((codes[:offset] == 99).all() and (codes[offset + n:] == 99).all())
        assert bool((xh[:offset] == 12345).all() and (xh[offset + n:] == 12345).all())
        assert bool((scales[:offset] == -5.0).all() and (scales[offset + batch * D:] == -5.0).all())
    with pytest.raises(kvq.KvqError):
        kvq.kvq_quantize_t(7, xd, scales, codes, batch, N, D)


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_sixteen_bit_quantize_every_finite_input_against_many_scales(fmt):
    """The 16-bit quantize kernel forms x / scale as a product with an fp64 reciprocal (provably the same
    fp32 quotient).  Every finite fp16 / bf16 value against 1024 scales spread over the whole fp32 range --
    subnormal, tiny, huge, negative, zero, powers of two and their neighbours -- must give the oracle's
    codes, which come from the plain fp32 divide."""
    rng = np.random.default_rng(len(fmt))
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    expo = ((bits >> 10) & 31) if fmt == "f16" else ((bits >> 7) & 255)
    bits = bits[expo != (31 if fmt == "f16" else 255)]                        # finite values only
    N, D = bits.size, 1024
    s = (2.0 ** rng.uniform(-149, 127, D) * rng.uniform(1, 2, D)).astype(np.float32)
    s[:16] = [0.0, -0.25, 2.0 ** -149, 2.0 ** -140, 2.0 ** -126, 2.0 ** 127, 3.0e38, 1.0, 1.0 + 2.0 ** -23,
              1.0 - 2.0 ** -24, 1.0 / 127, 3.0, 1.0 / 3, 65504.0 / 127, 2.0 ** -24, 2.0 ** -14 / 127]
    s[16:272] = (np.abs(oracle.widen16(bits, fmt)[rng.integers(0, N, 256)]) / np.float32(127)).astype(np.float32)
    s[272:400] *= np.float32(-1)
    # scales that put some input within an ulp of a .5 tie: |x0| / (k + 0.5)
    x0 = np.abs(oracle.widen16(bits, fmt)[rng.integers(0, N, 512)])
    s[400:912] = (x0 / (rng.integers(0, 127, 512).astype(np.float32) + np.float32(0.5))).astype(np.float32)
    x16 = np.ascontiguousarray(np.broadcast_to(bits[:, None], (N, D)))
    q_ref = oracle.quantize(oracle.widen16(x16, fmt), s)
    dt = kvq.DTYPE_F16 if fmt == "f16" else kvq.DTYPE_BF16
    xd = torch.from_numpy(x16.view(np.int16).reshape(-1)).cuda()
    sd = torch.from_numpy(s).cuda()
    codes = torch.full((N * D,), 99, dtype=torch.int8, device="cuda")
    kvq.kvq_quantize_t(dt, xd, sd, codes, 1, N, D)
    assert_bits_equal(codes.cpu().numpy().reshape(N, D), q_ref, "%s codes, all inputs x 1024 scales" % fmt)


def test_typed_calls_forward_fp32():
    x = W.generate(1)[0]
    g = Gpu(x)
    kvq.kvq_absmax_scales_t(kvq.DTYPE_F32, g.x, g.scales, 1, g.N, g.D)
    kvq.kvq_quantize_t(kvq.DTYPE_F32, g.x, g.scales, g.codes, 1, g.N, g.D)
    kvq.kvq_dequantize_t(kvq.DTYPE_F32, g.codes, g.scales, g.xh, 1, g.N, g.D)
    s_ref = oracle.compute_scales(x)
    q_ref = oracle.quantize(x, s_ref)
    assert_bits_equal(g.scales.cpu().numpy(), s_ref, "scales")
    assert_bits_equal(g.codes.cpu().numpy().reshape(g.N, g.D), q_ref, "codes")
    assert_bits_equal(g.xh.cpu().numpy().reshape(g.N, g.D), oracle.dequantize(q_ref, s_ref), "x_hat")


FUSED_SHAPES = [(7, 512, 128), (3, 1000, 64), (2, 16, 4096), (5, 17, 20), (1, 16384, 4), (1, 16385, 4),
                (4, 2048, 32), (9, 1, 8), (2, 513, 128), (1, 65, 1024), (300, 64, 64),
                # slabs cut into column tiles of a few 16-byte groups, all rows in one workgroup: slab counts that
                # do and do not fill the eight XCD queues, ragged row counts, tiles that overhang the last channel
                (3, 4096, 128), (9, 3000, 64), (1, 2048, 256), (5, 1500, 1000), (2, 4, 8192), (10, 4096, 16),
                (17, 4095, 20), (8, 1025, 136), (1, 4097, 128), (2, 700, 4100),
                # 2049 to 4096 rows: a 32-channel column tile in the registers and LDS of a persistent workgroup;
                # more tiles than workgroups, quads of tiles with empty places, one row past the register-only form
                (70, 4096, 128), (33, 3100, 260), (1, 2049, 128), (2, 4096, 36), (5, 2500, 1000), (600, 2050, 8),
                # the same with tiles of 64, 128 and 256 channels (1025 to 2048, 513 to 1024, 257 to 512 rows)
                (140, 2000, 128), (300, 1024, 128), (150, 512, 512), (7, 1900, 72), (3, 600, 1028), (2, 300, 2048)]


@pytest.mark.parametrize("shape", FUSED_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_single_pass_fused_slabs(shape):
    """Slabs at, below and just above what one workgroup's registers hold, whole or cut by column tile."""
    rng = np.random.default_rng(sum(shape))
    x = make_matrix(rng, *shape)
    s_ref = oracle.compute_scales(x)
    q_ref = oracle.quantize(x, s_ref)
    saved = (kvq.kvq_get_option(kvq.OPT_FUSED_MIN_LANES), kvq.kvq_get_option(kvq.OPT_FUSED_MAX_ROWS),
             kvq.kvq_get_option(kvq.OPT_FUSED_TALL))
    try:
        # the defaults; the narrowest column tiles with every register depth; wide tiles only; the persistent
        # form without its workgroups waiting for each other, wherever its tiles are at least half full, never
        for min_lanes, max_rows, tall in (saved, (4, 16, 1), (4, 8, 1), (4, 4, 1), (64, 0, 1), (saved[0], saved[1], 2),
                                         (saved[0], saved[1], 3), (saved[0], saved[1], 0)):
            kvq.kvq_set_option(kvq.OPT_FUSED_MIN_LANES, min_lanes)
            kvq.kvq_set_option(kvq.OPT_FUSED_MAX_ROWS, max_rows)
            kvq.kvq_set_option(kvq.OPT_FUSED_TALL, tall)
            g = Gpu(x)
            s_f, q_f = g.quantize_fused()
            what = "(min lanes %d, rows %d, tall %d)" % (min_lanes, max_rows, tall)
            assert_bits_equal(s_f, s_ref, "fused scales " + what)
            assert_bits_equal(q_f, q_ref, "fused codes " + what)
            assert g.guards_intact(), "fused wrote outside its buffers " + what
    finally:
        kvq.kvq_set_option(kvq.OPT_FUSED_MIN_LANES, saved[0])
        kvq.kvq_set_option(kvq.OPT_FUSED_MAX_ROWS, saved[1])
        kvq.kvq_set_option(kvq.OPT_FUSED_TALL, saved[2])


# ------------------------------------------------------------------ every launch shape, same bits
OPT_KEYS = (kvq.OPT_CODEC_WIDTH, kvq.OPT_CODEC_UNROLL, kvq.OPT_BLOCKS_PER_CU, kvq.OPT_NONTEMPORAL,
            kvq.OPT_BLOCK_THREADS, kvq.OPT_PASSES_PER_BLOCK)


def test_all_kernel_variants_give_identical_results():
    """Cross-variant consistency: lane width, unroll, workgroup size, one-shot or walking
    workgroups, cache hints -- none of them may change a bit."""
    rng = np.random.default_rng(5)
    x = make_matrix(rng, 2, 515, 272)
    s_ref = oracle.compute_scales(x)
    q_ref = oracle.quantize(x, s_ref)
    xh_ref = oracle.dequantize(q_ref, s_ref)
    saved = [kvq.kvq_get_option(k) for k in OPT_KEYS]
    try:
        combos = list(itertools.product((4, 8, 16), (0, 1, 2, 4, 8), (8,), (0, 1), (0,), (1,)))
        combos += list(itertools.product((4,), (2,), (1, 8), (1,), (64, 128, 256, 512), (0, 1, 3)))
        for combo in combos:
            for k, v in zip(OPT_KEYS, combo):
                kvq.kvq_set_option(k, v)
            g = Gpu(x)
            assert_bits_equal(g.absmax_scales(), s_ref, "scales %r" % (combo,))
            assert_bits_equal(g.quantize(), q_ref, "codes %r" % (combo,))
            assert_bits_equal(g.dequantize(), xh_ref, "x_hat %r" % (combo,))
            assert g.guards_intact(), combo
    finally:
        for k, v in zip(OPT_KEYS, saved):
            kvq.kvq_set_option(k, v)


ABSMAX_KEYS = (kvq.OPT_ABSMAX_SPAN, kvq.OPT_ABSMAX_BLOCKS_PER_CU, kvq.OPT_ABSMAX_UNROLL)


@pytest.mark.parametrize("shape", [(1, 3000, 8192), (3, 517, 2048), (1, 40000, 128), (700, 33, 64), (2, 9, 4100),
                                   (1, 70, 1 << 20)],
                         ids=lambda v: "x".join(map(str, v)))
def test_scales_do_not_depend_on_how_rows_are_chunked(shape):
    """The scale reduction splits a slab's rows over workgroups and merges their maxima through a workspace
    of fixed size.  Lanes spanning 1..8 column groups, 1..16 workgroups per compute unit (one chunk per slab
    up to hundreds; for the 2^20-channel matrix more chunks than the workspace holds, so they are merged
    down) and every unroll must give the oracle's bits, for fp32 and for 16-bit inputs."""
    batch, N, D = shape
    rng = np.random.default_rng(N + D)
    x = make_matrix(rng, batch, N, D)
    s_ref = oracle.compute_scales(x)
    x16 = x.astype(np.float16)
    s16_ref = oracle.compute_scales(x16.astype(np.float32))
    gx = torch.from_numpy(x.reshape(-1)).cuda()
    gx16 = torch.from_numpy(x16.reshape(-1)).cuda()
    scales = torch.empty(batch * D, dtype=torch.float32, device="cuda")
    saved = [kvq.kvq_get_option(k) for k in ABSMAX_KEYS]
    try:
        for combo in itertools.product((1, 2, 8), (1, 4, 16), (4, 16)):
            for k, v in zip(ABSMAX_KEYS, combo):
                kvq.kvq_set_option(k, v)
            scales.fill_(-1.0)
            kvq.kvq_absmax_scales(gx, scales, batch, N, D)
            assert_bits_equal(scales.cpu().numpy().reshape(s_ref.shape), s_ref, "fp32 scales %r" % (combo,))
            scales.fill_(-1.0)
            kvq.kvq_absmax_scales_t(kvq.DTYPE_F16, gx16, scales, batch, N, D)
            assert_bits_equal(scales.cpu().numpy().reshape(s16_ref.shape), s16_ref, "fp16 scales %r" % (combo,))
    finally:
        for k, v in zip(ABSMAX_KEYS, saved):
            kvq.kvq_set_option(k, v)


# ------------------------------------------------------------------ numerics corner cases
def test_ties_near_ties_and_clipping_with_given_scales():
    """Quotients on and next to .5 ties, scales that clip, tiny, huge, zero and negative scales."""
    rng = np.random.default_rng(17)
    N, D = 4096, 64
    s = np.exp(rng.uniform(-3, 3, D)).astype(np.float32)
    s[0], s[1], s[2], s[3] = 2.0 ** -140, 2.0 ** 120, 1e-3, 3.0      # subnormal, huge, clipping, coarse
    s[4] = 0.0
    s[5] = -0.25                                                       # a negative scale is still a divisor
    k = rng.integers(-130, 131, (N, D)).astype(np.float64) + 0.5
    x = (k * s.astype(np.float64)).astype(np.float32)                  # quotient within an ulp of a tie
    x[::3] = np.nextafter(x[::3], np.float32(np.inf))
    x[1::3] = np.nextafter(x[1::3], np.float32(-np.inf))
    x[:, 0] = (rng.integers(-200, 200, N) * 2.0 ** -141).astype(np.float32)
    x[:, 1] = (rng.standard_normal(N) * 2.0 ** 125).astype(np.float32)
    g = Gpu(x)
    g.set_scales(s)
    q_ref = oracle.quantize(x, s)
    assert_bits_equal(g.quantize()[0], q_ref, "codes near ties")
    assert_bits_equal(g.dequantize()[0], oracle.dequantize(q_ref, s), "x_hat")
    assert len(np.unique(q_ref)) == 255


def test_subnormal_inputs_and_scales():
    tiny = np.float32(2.0 ** -149)
    x = np.zeros((64, 16), dtype=np.float32)
    x[:, 0] = (np.arange(64) - 32) * tiny * 3          # absmax 96 ulp -> scale rounds to 1 ulp (subnormal)
    x[:, 1] = (np.arange(64) % 7) * tiny               # absmax 6 ulp  -> scale underflows to 0
    x[:, 2] = 1.0
    x[1:, 2] = tiny
    x[:, 3] = np.float32(3e38)
    x[::2, 3] = np.float32(-1e-38)
    g = full_round_trip_check(x, tag="subnormal")
    s = g.scales.cpu().numpy()
    assert s[0] == tiny and s[1] == 0.0


def test_identity_metrics_are_zero_on_gpu():
    x = W.generate(1)[0]
    g = Gpu(x)
    g.xh.copy_(g.x)
    assert g.roundtrip_error(from_codes=False) == (0.0, 0.0)
    assert g.attn_score_error(W.queries(1), from_codes=False) == 0.0


def test_results_are_deterministic_run_to_run():
    x = W.generate(2)[0]
    g = Gpu(x)
    g.absmax_scales()
    g.quantize()
    g.dequantize()
    first = (g.scales.clone(), g.codes.clone(), g.roundtrip_error(False), g.roundtrip_error(True),
             g.attn_score_error(W.queries(2), False))
    for _ in range(3):
        g.absmax_scales()
        g.quantize()
        assert torch.equal(g.scales, first[0]) and torch.equal(g.codes, first[1])
        assert g.roundtrip_error(False) == first[2] and g.roundtrip_error(True) == first[3]
        assert g.attn_score_error(W.queries(2), False) == first[4]


def test_stale_contents_of_the_scale_buffer_and_workspace_do_not_survive():
    """Whatever the scale buffer held, and whatever an earlier, larger reduction left in the workspace of
    per-chunk maxima, the scales are those of the matrix at hand."""
    big = make_matrix(np.random.default_rng(3), 1, 40000, 128) * np.float32(1e6)   # many row chunks, huge maxima
    gb = Gpu(big)
    assert_bits_equal(gb.absmax_scales(), oracle.compute_scales(big), "large matrix first")
    for cfg in (1, 2):
        x = W.generate(cfg)[0]
        g = Gpu(x)
        g.scales.fill_(1e30)
        assert_bits_equal(g.absmax_scales()[0], oracle.compute_scales(x), "scales after stale contents")


def test_works_on_a_non_default_stream():
    x = W.generate(1)[0]
    s_ref = oracle.compute_scales(x)
    q_ref = oracle.quantize(x, s_ref)
    g = Gpu(x)
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        h = st.cuda_stream
        kvq.kvq_absmax_scales(g.x, g.scales, 1, g.N, g.D, stream=h)
        kvq.kvq_quantize(g.x, g.scales, g.codes, 1, g.N, g.D, stream=h)
        kvq.kvq_dequantize(g.codes, g.scales, g.xh, 1, g.N, g.D, stream=h)
        kvq.kvq_roundtrip_error(g.x, g.xh, None, None, 1, g.N, g.D, g.sumsq, g.maxabs, stream=h)
    st.synchronize()
    assert_bits_equal(g.codes.cpu().numpy().reshape(g.N, g.D), q_ref, "codes on side stream")
    xh_ref = oracle.dequantize(q_ref, s_ref)
    ss_ref, mx_ref = oracle.roundtrip_error(x, xh_ref)
    assert float(g.sumsq.item()) == pytest.approx(ss_ref, rel=REL) and np.float32(g.maxabs.item()) == mx_ref


def test_streams_do_not_share_scratch():
    """The scale reduction and the error kernels keep partial results in a per-stream workspace.  Four
    streams work on four different matrices at once, several rounds without synchronising in between;
    every stream must end with its own matrix's oracle results."""
    rng = np.random.default_rng(23)
    shapes = [(1, 30000, 256), (4, 6000, 128), (1, 2500, 4096), (2, 9000, 512)]
    xs = [(make_matrix(rng, *sh) * np.float32(10.0 ** i)).astype(np.float32) for i, sh in enumerate(shapes)]
    gs = [Gpu(x) for x in xs]
    streams = [torch.cuda.Stream() for _ in xs]
    torch.cuda.synchronize()
    for _ in range(5):
        for g, st in zip(gs, streams):
            h = st.cuda_stream
            kvq.kvq_absmax_scales(g.x, g.scales, g.batch, g.N, g.D, stream=h)
            kvq.kvq_quantize(g.x, g.scales, g.codes, g.batch, g.N, g.D, stream=h)
            kvq.kvq_roundtrip_error(g.x, None, g.codes, g.scales, g.batch, g.N, g.D, g.sumsq, g.maxabs, stream=h)
    torch.cuda.synchronize()
    for x, g in zip(xs, gs):
        s_ref = oracle.compute_scales(x)
        q_ref = oracle.quantize(x, s_ref)
        assert_bits_equal(g.scales.cpu().numpy().reshape(s_ref.shape), s_ref, "scales %r" % (g.shape,))
        assert_bits_equal(g.codes.cpu().numpy().reshape(q_ref.shape), q_ref, "codes %r" % (g.shape,))
        ss_ref, mx_ref = oracle.roundtrip_error(x, oracle.dequantize(q_ref, s_ref))
        assert float(g.sumsq.item()) == pytest.approx(ss_ref, rel=REL) and np.float32(g.maxabs.item()) == mx_ref


def test_a_streams_workspace_can_be_released_and_comes_back():
    x = make_matrix(np.random.default_rng(8), 1, 9000, 256)
    s_ref = oracle.compute_scales(x)
    g = Gpu(x)
    torch.cuda.synchronize()                        # the input copy ran on the default stream
    st = torch.cuda.Stream()
    h = st.cuda_stream
    kvq.kvq_release_stream(h)                       # nothing there yet: still OK
    kvq.kvq_prepare_stream(h)
    for _ in range(3):
        kvq.kvq_absmax_scales(g.x, g.scales, 1, g.N, g.D, stream=h)
        st.synchronize()
        assert_bits_equal(g.scales.cpu().numpy().reshape(s_ref.shape), s_ref, "scales")
        kvq.kvq_release_stream(h)                   # the next call allocates a fresh workspace
    kvq.kvq_release_stream(h)


# ------------------------------------------------------------------ 4-bit codes
def int4_round_trip(x, offset=0, given_scales=None):
    """kvq_*_int4 against the oracle's qmax = 7 functions: scales, packed bytes and x_hat bit-exact,
    and nothing written outside the buffers."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim == 2:
        x = x[None]
    batch, N, D = x.shape
    n = x.size
    dx = torch.empty(n + 64, dtype=torch.float32, device="cuda")
    xs = dx[offset:offset + n]
    xs.copy_(torch.from_numpy(x.reshape(-1)))
    ds = torch.full((batch * D + 64,), -5.0, dtype=torch.float32, device="cuda")
    ss = ds[offset:offset + batch * D]
    dp = torch.full((n // 2 + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    ps = dp[offset:offset + n // 2]
    dh = torch.full((n + 64,), 777.0, dtype=torch.float32, device="cuda")
    hs = dh[offset:offset + n]
    if given_scales is None:
        kvq.kvq_absmax_scales_int4(xs, ss, batch, N, D)
        s_ref = oracle.compute_scales_q(x, 7)
        assert_bits_equal(ss.cpu().numpy().reshape(batch, D), s_ref, "int4 scales")
    else:
        s_ref = np.ascontiguousarray(given_scales, dtype=np.float32).reshape(batch, D)
        ss.copy_(torch.from_numpy(s_ref.reshape(-1)))
    kvq.kvq_quantize_int4(xs, ss, ps, batch, N, D)
    q_ref = oracle.quantize_q(x, s_ref, 7)
    p_ref = oracle.pack_int4(q_ref)
    assert_bits_equal(ps.cpu().numpy().reshape(batch, N, D // 2), p_ref, "packed 4-bit codes")
    kvq.kvq_dequantize_int4(ps, ss, hs, batch, N, D)
    assert_bits_equal(hs.cpu().numpy().reshape(x.shape), oracle.dequantize(q_ref, s_ref), "int4 x_hat")
    torch.cuda.synchronize()
    assert bool((dp[:offset] == 0x5A).all() and (dp[offset + n // 2:] == 0x5A).all())
    assert bool((dh[:offset] == 777.0).all() and (dh[offset + n:] == 777.0).all())
    assert bool((ds[:offset] == -5.0).all() and (ds[offset + batch * D:] == -5.0).all())
    return q_ref


INT4_SHAPES = [(1, 1, 2), (1, 3, 6), (1, 64, 16), (3, 5, 18), (1, 100, 62), (2, 33, 66), (1, 300, 128),
               (2, 257, 1000), (1, 19, 4096), (1, 3, 4100), (1, 3, 4102), (5, 1, 272), (1, 2050, 8), (1, 1024, 64),
               (1, 4100, 256), (8, 515, 128)]


@pytest.mark.parametrize("shape", INT4_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_int4_ragged_shapes(shape):
    rng = np.random.default_rng(seed_of(shape))
    x = make_matrix(rng, *shape)
    if shape[2] >= 6 and shape[1] >= 4:          # exact ties at 4 bits: multiples of s/2 with absmax 7 s
        s = np.float32(0.5)
        x[:, :, 4] = (rng.integers(-13, 14, shape[:2]) * (s / 2)).astype(np.float32)
        x[:, 0, 4] = 7 * s
    q = int4_round_trip(x)
    assert np.abs(q).max() <= 7


@pytest.mark.parametrize("offset", [1, 2, 3, 4, 8])
def test_int4_unaligned_base_pointers(offset):
    rng = np.random.default_rng(offset)
    int4_round_trip(make_matrix(rng, 2, 70, 64), offset=offset)


def test_int4_config2_and_config3_slabs():
    q = int4_round_trip(W.generate(2)[0])
    assert set(np.unique(q).tolist()) == set(range(-7, 8))
    int4_round_trip(W.generate(3, slabs=(0, 40)))


def test_int4_ties_clipping_and_special_scales():
    rng = np.random.default_rng(23)
    N, D = 4096, 64
    s = np.exp(rng.uniform(-3, 3, D)).astype(np.float32)
    s[0], s[1], s[2], s[3], s[4], s[5] = 2.0 ** -140, 2.0 ** 120, 1e-3, 3.0, 0.0, -0.25
    k = rng.integers(-9, 10, (N, D)).astype(np.float64) + 0.5
    x = (k * s.astype(np.float64)).astype(np.float32)
    x[::3] = np.nextafter(x[::3], np.float32(np.inf))
    x[1::3] = np.nextafter(x[1::3], np.float32(-np.inf))
    x[:, 0] = (rng.integers(-20, 20, N) * 2.0 ** -141).astype(np.float32)
    x[:, 1] = (rng.standard_normal(N) * 2.0 ** 125).astype(np.float32)
    int4_round_trip(x, given_scales=s)


def test_int4_rejects_an_odd_channel_count():
    x = torch.zeros(15, dtype=torch.float32, device="cuda")
    s = torch.zeros(5, dtype=torch.float32, device="cuda")
    p = torch.zeros(8, dtype=torch.uint8, device="cuda")
    with pytest.raises(kvq.KvqError) as e:
        kvq.kvq_quantize_int4(x, s, p, 1, 3, 5)
    assert e.value.status == kvq.ERR_ARG
    with pytest.raises(kvq.KvqError) as e:
        kvq.kvq_dequantize_int4(p, s, x, 1, 3, 5)
    assert e.value.status == kvq.ERR_ARG


def test_int4_full_size_sampled_rows():
    """The 1B-element configuration in the launch shape the report times: scales of the whole matrix
    against the oracle, packed codes and x_hat on sampled row blocks."""
    c = W.CONFIGS[5]
    x = W.generate(5)[0]
    s_ref = oracle.compute_scales_q(x, 7)
    dx = torch.from_numpy(x).cuda()
    ds = torch.empty(c.D, dtype=torch.float32, device="cuda")
    dp = torch.empty((c.N, c.D // 2), dtype=torch.uint8, device="cuda")
    dh = torch.empty((c.N, c.D), dtype=torch.float32, device="cuda")
    kvq.kvq_absmax_scales_int4(dx, ds, 1, c.N, c.D)
    assert_bits_equal(ds.cpu().numpy(), s_ref, "int4 scales of the full matrix")
    kvq.kvq_quantize_int4(dx, ds, dp, 1, c.N, c.D)
    kvq.kvq_dequantize_int4(dp, ds, dh, 1, c.N, c.D)
    rows = 4096
    for r0 in (0, 37 * rows + 5, c.N - rows):
        q_ref = oracle.quantize_q(x[r0:r0 + rows], s_ref, 7)
        assert_bits_equal(dp[r0:r0 + rows].cpu().numpy(), oracle.pack_int4(q_ref), "packed rows %d" % r0)
        assert_bits_equal(dh[r0:r0 + rows].cpu().numpy(), oracle.dequantize(q_ref, s_ref), "x_hat rows %d" % r0)


# ------------------------------------------------------------------ streaming append
class GpuCache:
    """A device cache [batch, capacity, D] of codes + scales, driven through kvq_append."""

    def __init__(self, batch, capacity, D, offset=0):
        self.batch, self.cap, self.D, self.offset = batch, capacity, D, offset
        n = batch * capacity * D
        self._codes = torch.full((n + 64,), 55, dtype=torch.int8, device="cuda")
        self.codes = self._codes[offset:offset + n]
        self._scales = torch.full((batch * D + 64,), -5.0, dtype=torch.float32, device="cuda")
        self.scales = self._scales[offset:offset + batch * D]
        self.scales.zero_()
        self._prev = torch.full((batch * D + 64,), -6.0, dtype=torch.float32, device="cuda")
        self.prev = self._prev[offset:offset + batch * D]
        self.n = 0

    def append(self, x_np):
        x_np = np.ascontiguousarray(x_np, dtype=np.float32)
        m = x_np.shape[1]
        buf = torch.empty(x_np.size + 64, dtype=torch.float32, device="cuda")
        xs = buf[self.offset:self.offset + x_np.size]
        xs.copy_(torch.from_numpy(x_np.reshape(-1)))
        kvq.kvq_append(xs, self.scales, self.prev, self.codes, self.batch, self.n, m, self.cap, self.D)
        self.n += m

    def state(self):
        return (self.codes.cpu().numpy().reshape(self.batch, self.cap, self.D),
                self.scales.cpu().numpy().reshape(self.batch, self.D),
                self.prev.cpu().numpy().reshape(self.batch, self.D))

    def guards_intact(self):
        o, n, ns = self.offset, self.batch * self.cap * self.D, self.batch * self.D
        return bool((self._codes[:o] == 55).all() and (self._codes[o + n:] == 55).all() and
                    (self._scales[:o] == -5.0).all() and (self._scales[o + ns:] == -5.0).all() and
                    (self._prev[:o] == -6.0).all() and (self._prev[o + ns:] == -6.0).all())


def growing_tokens(rng, batch, N, D):
    """Channels 0.. grow at different moments; channel 1 is zero, channel 4 is fixed by its first token."""
    x = make_matrix(rng, batch, N, D)
    ramp = np.linspace(0.2, 3.0, N)[None, :]
    x[:, :, 0] *= ramp
    if D >= 8:
        x[:, :, 7] *= ramp ** 2
        x[:, :, 4] = rng.uniform(-1, 1, (batch, N))
        x[:, 0, 4] = 2.0
    if N > 40:
        x[0, 40, D - 1] = 1e4                    # one late outlier: a single growth event in slab 0
    return x


APPEND_CASES = [((1, 64, 64), (1, 1, 1, 5, 16, 17, 23)), ((3, 300, 128), (17, 1, 100, 1, 1, 64, 116)),
                ((2, 40, 20), (1, 16, 1, 22)), ((1, 33, 3), (1, 1, 31)), ((2, 50, 65), (20, 1, 29)),
                ((4, 2100, 256), (2048, 1, 1, 50)), ((1, 9, 4100), (1, 3, 5)), ((6, 48, 8), (48,))]


@pytest.mark.parametrize("shape,chunks", APPEND_CASES, ids=lambda v: "x".join(map(str, v)))
@pytest.mark.parametrize("offset", [0, 1])
def test_streaming_append_matches_oracle(shape, chunks, offset):
    batch, cap, D = shape
    rng = np.random.default_rng(seed_of(shape, offset))
    N = sum(chunks)
    assert N <= cap
    x = growing_tokens(rng, batch, N, D)
    g = GpuCache(batch, cap, D, offset)
    ref_codes = np.full((batch, cap, D), 55, dtype=np.int8)
    ref_scales = np.zeros((batch, D), dtype=np.float32)
    n, grown_total = 0, 0
    for m in chunks:
        g.append(x[:, n:n + m])
        ref_codes, new_scales, ref_prev = oracle.append(ref_codes, ref_scales, n, x[:, n:n + m])
        grown_total += int(((new_scales > ref_scales) & (n > 0)).sum())
        ref_scales, n = new_scales, n + m
        codes, scales, prev = g.state()
        assert_bits_equal(scales, ref_scales, "scales after %d tokens" % n)
        assert_bits_equal(prev, ref_prev, "previous scales after %d tokens" % n)
        assert_bits_equal(codes, ref_codes, "cache after %d tokens" % n)
    assert g.guards_intact()
    assert_bits_equal(ref_scales, oracle.compute_scales(x), "running scales = batch scales")
    if len(chunks) > 1:
        assert grown_total > 0            # the requantization path was exercised


def test_streaming_append_decode_step_on_a_full_size_cache():
    """[256 x 4096 x 128] (config 3's cache), 4095 tokens in place, one more arrives: a few slabs
    grow, most do not; whole cache against the oracle."""
    c = W.CONFIGS[3]
    x = W.generate(3)
    n_old = c.N - 1
    s_old = oracle.compute_scales(x[:, :n_old])
    cache = np.full((c.batch, c.N, c.D), 55, dtype=np.int8)
    cache[:, :n_old] = oracle.quantize(np.ascontiguousarray(x[:, :n_old]), s_old)
    tok = np.ascontiguousarray(x[:, n_old:])
    tok[3, 0, 5] = 4 * s_old[3, 5] * 127            # planted growth: one channel in slab 3,
    tok[200, 0, :] = -2 * s_old[200] * 127          # and every channel of slab 200
    g = GpuCache(c.batch, c.N, c.D)
    g.codes.copy_(torch.from_numpy(cache.reshape(-1)))
    g.scales.copy_(torch.from_numpy(s_old.reshape(-1)))
    g.n = n_old
    g.append(tok)
    ref_codes, ref_scales, ref_prev = oracle.append(cache, s_old, n_old, tok)
    codes, scales, prev = g.state()
    assert_bits_equal(scales, ref_scales, "scales")
    assert_bits_equal(prev, ref_prev, "previous scales")
    assert_bits_equal(codes, ref_codes, "cache")
    grew = ref_scales > s_old
    assert grew[3, 5] and grew[200].all() and grew.sum() < 0.2 * grew.size


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
@pytest.mark.parametrize("shape,chunks", [((3, 300, 128), (17, 1, 100, 1, 1, 64, 116)), ((2, 40, 20), (1, 16, 1, 22)),
                                          ((1, 33, 3), (1, 1, 31)), ((4, 2100, 256), (2048, 1, 1, 50)),
                                          ((1, 9, 4100), (1, 3, 5)), ((2, 50, 65), (20, 1, 29))],
                         ids=lambda v: "x".join(map(str, v)))
@pytest.mark.parametrize("offset", [0, 1])
def test_streaming_append_of_sixteen_bit_tokens(shape, chunks, offset, fmt):
    """kvq_append_t: new tokens arrive as fp16 / bf16; the cache must be what the oracle's append gives
    for the widened tokens, bit for bit, through decode steps, prefill chunks and misaligned buffers."""
    batch, cap, D = shape
    rng = np.random.default_rng(seed_of(shape, offset, fmt))
    N = sum(chunks)
    x16 = oracle.narrow16(np.clip(growing_tokens(rng, batch, N, D), -60000, 60000), fmt)
    xw = oracle.widen16(x16, fmt)
    dt = kvq.DTYPE_F16 if fmt == "f16" else kvq.DTYPE_BF16
    g = GpuCache(batch, cap, D, offset)
    ref_codes = np.full((batch, cap, D), 55, dtype=np.int8)
    ref_scales = np.zeros((batch, D), dtype=np.float32)
    n, grown_total = 0, 0
    for m in chunks:
        tok = np.ascontiguousarray(x16[:, n:n + m])
        buf = torch.zeros(tok.size + 64, dtype=torch.int16, device="cuda")
        xs = buf[offset:offset + tok.size]
        xs.copy_(torch.from_numpy(tok.view(np.int16).reshape(-1)))
        kvq.kvq_append_t(dt, xs, g.scales, g.prev, g.codes, batch, n, m, cap, D)
        ref_codes, new_scales, ref_prev = oracle.append(ref_codes, ref_scales, n, np.ascontiguousarray(xw[:, n:n + m]))
        grown_total += int(((new_scales > ref_scales) & (n > 0)).sum())
        ref_scales, n = new_scales, n + m
        codes, scales, prev = g.state()
        assert_bits_equal(scales, ref_scales, "scales after %d tokens" % n)
        assert_bits_equal(prev, ref_prev, "previous scales after %d tokens" % n)
        assert_bits_equal(codes, ref_codes, "cache after %d tokens" % n)
    assert g.guards_intact()
    assert grown_total > 0
    # fp32 through the typed entry point is the fp32 call
    g32 = GpuCache(batch, cap, D, offset)
    buf = torch.zeros(xw[:, :chunks[0]].size + 64, dtype=torch.float32, device="cuda")
    xs = buf[offset:offset + xw[:, :chunks[0]].size]
    xs.copy_(torch.from_numpy(np.ascontiguousarray(xw[:, :chunks[0]]).reshape(-1)))
    kvq.kvq_append_t(kvq.DTYPE_F32, xs, g32.scales, g32.prev, g32.codes, batch, 0, chunks[0], cap, D)
    want, _, _ = oracle.append(np.full((batch, cap, D), 55, dtype=np.int8), np.zeros((batch, D), np.float32), 0,
                               np.ascontiguousarray(xw[:, :chunks[0]]))
    assert_bits_equal(g32.state()[0], want, "fp32 through kvq_append_t")
    with pytest.raises(kvq.KvqError) as e:
        kvq.kvq_append_t(9, xs, g32.scales, g32.prev, g32.codes, batch, 0, 1, cap, D)
    assert e.value.status == kvq.ERR_ARG


@pytest.mark.parametrize("shape,chunks", [((3, 300, 128), (17, 1, 100, 1, 1, 64, 116)), ((2, 40, 20), (1, 16, 1, 22)),
                                          ((1, 33, 2), (1, 1, 31)), ((4, 2100, 256), (2048, 1, 1, 50)),
                                          ((1, 9, 4100), (1, 3, 5)), ((2, 50, 66), (20, 1, 29)), ((6, 48, 8), (48,))],
                         ids=lambda v: "x".join(map(str, v)))
@pytest.mark.parametrize("offset", [0, 1])
def test_streaming_append_onto_a_four_bit_cache(shape, chunks, offset):
    """kvq_append_int4 against the oracle's append with the range [-7, 7]: scales, previous scales and the
    packed cache bit for bit through decode steps and prefill chunks, aligned and misaligned; bytes of
    rows beyond the valid ones untouched."""
    batch, cap, D = shape
    rng = np.random.default_rng(seed_of(shape, offset, 4))
    N = sum(chunks)
    x = growing_tokens(rng, batch, N, D)
    nb = batch * cap * D // 2
    pbuf = torch.full((nb + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    packed = pbuf[offset:offset + nb]
    sbuf = torch.full((batch * D + 64,), -5.0, dtype=torch.float32, device="cuda")
    scales = sbuf[offset:offset + batch * D]
    scales.zero_()
    vbuf = torch.full((batch * D + 64,), -6.0, dtype=torch.float32, device="cuda")
    prev = vbuf[offset:offset + batch * D]
    ref_codes = np.zeros((batch, cap, D), dtype=np.int8)
    ref_scales = np.zeros((batch, D), dtype=np.float32)
    n, grown_total = 0, 0
    for m in chunks:
        tok = np.ascontiguousarray(x[:, n:n + m])
        buf = torch.empty(tok.size + 64, dtype=torch.float32, device="cuda")
        xs = buf[offset:offset + tok.size]
        xs.copy_(torch.from_numpy(tok.reshape(-1)))
        kvq.kvq_append_int4(xs, scales, prev, packed, batch, n, m, cap, D)
        ref_codes, new_scales, ref_prev = oracle.append_q(ref_codes, ref_scales, n, tok, 7)
        grown_total += int(((new_scales > ref_scales) & (n > 0)).sum())
        ref_scales, n = new_scales, n + m
        assert_bits_equal(scales.cpu().numpy().reshape(batch, D), ref_scales, "scales after %d tokens" % n)
        assert_bits_equal(prev.cpu().numpy().reshape(batch, D), ref_prev, "previous scales after %d tokens" % n)
        got = packed.cpu().numpy().reshape(batch, cap, D // 2)
        want = oracle.pack_int4(np.ascontiguousarray(ref_codes[:, :n]))
        assert np.array_equal(got[:, :n], want), "cache after %d tokens" % n
        assert (got[:, n:] == 0x5A).all(), "rows beyond the valid ones"
    assert bool((pbuf[:offset] == 0x5A).all() and (pbuf[offset + nb:] == 0x5A).all())
    assert bool((sbuf[:offset] == -5.0).all() and (sbuf[offset + batch * D:] == -5.0).all())
    assert bool((vbuf[:offset] == -6.0).all() and (vbuf[offset + batch * D:] == -6.0).all())
    if len(chunks) > 1:
        assert grown_total > 0
    with pytest.raises(kvq.KvqError) as e:
        kvq.kvq_append_int4(xs, scales, prev, packed, batch, 0, 1, cap, D + 1)
    assert e.value.status == kvq.ERR_ARG


def test_append_requantization_on_and_next_to_ties():
    """The requantization forms (float)code * s_old / s_new without a divide instruction.  Every code value
    in every channel, with new scales that are 2 s_old up to a rounding error (quotients on and within an ulp
    of .5 ties), a little above s_old (quotients just under the integers) and far above: the oracle, which
    divides in fp32, must be matched bit for bit -- for the 8-bit and the 4-bit cache."""
    rng = np.random.default_rng(77)
    D = 512
    for qmax, fn in ((127, "int8"), (7, "int4")):
        n_old = 2 * qmax + 1
        cap = n_old + 1
        s_old = np.exp(rng.uniform(-20, 20, (1, D))).astype(np.float32)
        cache = np.zeros((1, cap, D), dtype=np.int8)
        cache[0, :n_old] = np.arange(-qmax, qmax + 1, dtype=np.int8)[:, None]
        tok = np.zeros((1, 1, D), dtype=np.float32)
        third = D // 3
        tok[0, 0, :third] = (s_old[0, :third] * np.float32(2 * qmax)) * rng.choice([-1, 1], third).astype(np.float32)
        tok[0, 0, :third] *= 1 + rng.integers(0, 4, third).astype(np.float32) * np.float32(2.0 ** -23)   # s_new = 2 s_old (1 + k ulp)
        tok[0, 0, third:2 * third] = s_old[0, third:2 * third] * np.float32(qmax) * (
            1 + rng.integers(1, 64, third).astype(np.float32) * np.float32(2.0 ** -22))
        tok[0, 0, 2 * third:] = s_old[0, 2 * third:] * np.float32(qmax) * np.exp(rng.uniform(0, 8, D - 2 * third)).astype(np.float32)
        ref_codes, ref_scales, _ = oracle.append_q(cache, s_old, n_old, tok, qmax)
        assert (ref_scales > s_old).all()
        scales = torch.from_numpy(s_old.reshape(-1)).cuda()
        prev = torch.empty_like(scales)
        xs = torch.from_numpy(tok.reshape(-1)).cuda()
        if qmax == 127:
            codes = torch.from_numpy(cache.reshape(-1)).cuda()
            kvq.kvq_append(xs, scales, prev, codes, 1, n_old, 1, cap, D)
            got = codes.cpu().numpy().reshape(1, cap, D)
            assert_bits_equal(got, ref_codes, "8-bit cache")
        else:
            packed = torch.from_numpy(oracle.pack_int4(cache).reshape(-1)).cuda()
            kvq.kvq_append_int4(xs, scales, prev, packed, 1, n_old, 1, cap, D)
            got = packed.cpu().numpy().reshape(1, cap, D // 2)
            assert np.array_equal(got, oracle.pack_int4(ref_codes)), "4-bit cache"
        assert_bits_equal(scales.cpu().numpy().reshape(1, D), ref_scales, fn + " scales")


def test_streaming_append_argument_errors():
    g = GpuCache(1, 8, 4)
    x = torch.zeros(4 * 4, dtype=torch.float32, device="cuda")
    for args, status in ((dict(n_old=6, m=3), kvq.ERR_ARG), (dict(n_old=-1, m=1), kvq.ERR_SHAPE),
                         (dict(n_old=0, m=0), kvq.ERR_SHAPE), (dict(n_old=0, m=9), kvq.ERR_ARG)):
        with pytest.raises(kvq.KvqError) as e:
            kvq.kvq_append(x, g.scales, g.prev, g.codes, 1, args["n_old"], args["m"], 8, 4)
        assert e.value.status == status
    with pytest.raises(kvq.KvqError) as e:
        kvq.kvq_append(x, g.scales, g.scales, g.codes, 1, 0, 1, 8, 4)
    assert e.value.status == kvq.ERR_ARG
    assert bool((g.codes == 55).all())


# ------------------------------------------------------------------ HIP graph capture
def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """The library enqueues only kernels (no memsets, no allocations once the per-stream workspace of
    the error kernels exists), so a whole step can be captured once and replayed.  Each replay, with
    eager work and synchronisation in between, must reproduce the eager results bit for bit."""
    rng = np.random.default_rng(5)
    batch, N, D = 3, 700, 128
    xs = [make_matrix(rng, batch, N, D) for _ in range(3)]
    g = Gpu(xs[0])
    packed = torch.zeros(batch * N * D // 2, dtype=torch.uint8, device="cuda")
    s4 = torch.zeros(batch * D, dtype=torch.float32, device="cuda")
    qs = torch.from_numpy(rng.standard_normal((5, D)).astype(np.float32)).cuda()
    mean2 = torch.zeros(1, dtype=torch.float64, device="cuda")

    def step():
        kvq.kvq_absmax_scales(g.x, g.scales, batch, N, D)
        kvq.kvq_quantize(g.x, g.scales, g.codes, batch, N, D)
        kvq.kvq_dequantize(g.codes, g.scales, g.xh, batch, N, D)
        kvq.kvq_roundtrip_error(g.x, g.xh, None, None, batch, N, D, g.sumsq, g.maxabs)
        kvq.kvq_absmax_scales_int4(g.x, s4, batch, N, D)
        kvq.kvq_quantize_int4(g.x, s4, packed, batch, N, D)
        # the score error of the first slab, both forms (rows of 128 channels: the bf16 matrix-core kernels)
        kvq.kvq_attn_score_error(qs, 5, g.x, g.xh, None, None, N, D, g.mean)
        kvq.kvq_attn_score_error(qs, 5, g.x, None, g.codes, g.scales, N, D, mean2)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (g.scales, g.codes, g.xh, g.sumsq, g.maxabs, s4, packed, g.mean, mean2)]

    side = torch.cuda.Stream()
    kvq.kvq_prepare_stream(side.cuda_stream)    # this stream's workspace exists before the capture
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for x_np in xs[1:] + xs[:1]:
        g.x.copy_(torch.from_numpy(x_np.reshape(-1)))
        step()
        want = snapshot()
        for t in (g.scales, g.xh, s4):
            t.fill_(-1.0)
        g.codes.fill_(77)
        packed.fill_(0x33)
        g.mean.fill_(-1.0)
        mean2.fill_(-1.0)
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for a, b in zip(got, want):
            assert torch.equal(a, b)
    s_ref = oracle.compute_scales(xs[0])
    assert_bits_equal(g.scales.cpu().numpy().reshape(batch, D), s_ref, "scales after the last replay")
    assert_bits_equal(g.codes.cpu().numpy().reshape(batch, N, D), oracle.quantize(xs[0], s_ref), "codes after replay")


def test_fused_call_on_tall_slabs_can_be_captured_and_replayed():
    """kvq_quantize_fused on slabs of 2049 to 4096 rows: its workgroups count themselves in and out of a
    few counters in the stream's workspace and leave them at zero, so the launch can be captured once and
    replayed; more tiles than workgroups, so some take a second tile."""
    rng = np.random.default_rng(6)
    batch, N, D = 70, 2100, 128
    xs = [make_matrix(rng, batch, N, D) for _ in range(2)]
    g = Gpu(xs[0])
    side = torch.cuda.Stream()
    kvq.kvq_prepare_stream(side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        kvq.kvq_quantize_fused(g.x, g.scales, g.codes, batch, N, D)
    for x_np in (xs[1], xs[0], xs[1]):
        g.x.copy_(torch.from_numpy(x_np.reshape(-1)))
        g.scales.fill_(-1.0)
        g.codes.fill_(77)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        s_ref = oracle.compute_scales(x_np)
        assert_bits_equal(g.scales.cpu().numpy().reshape(batch, D), s_ref, "scales after a replay")
        assert_bits_equal(g.codes.cpu().numpy().reshape(batch, N, D), oracle.quantize(x_np, s_ref), "codes after a replay")
        # the same call eagerly, on the default stream (its own workspace)
        s_f, q_f = g.quantize_fused()
        assert_bits_equal(s_f, s_ref, "scales, eager")
        assert g.guards_intact()


# ------------------------------------------------------------------ FP8 (E4M3) codes
def fp8_round_trip(x, offset=0, given_scales=None):
    """kvq_*_fp8 against the oracle: scales (absmax / 448), E4M3 codes and x_hat bit-exact."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim == 2:
        x = x[None]
    batch, N, D = x.shape
    n = x.size
    dx = torch.empty(n + 64, dtype=torch.float32, device="cuda")
    xs = dx[offset:offset + n]
    xs.copy_(torch.from_numpy(x.reshape(-1)))
    ds = torch.full((batch * D + 64,), -5.0, dtype=torch.float32, device="cuda")
    ss = ds[offset:offset + batch * D]
    dc = torch.full((n + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    cs = dc[offset:offset + n]
    dh = torch.full((n + 64,), 777.0, dtype=torch.float32, device="cuda")
    hs = dh[offset:offset + n]
    if given_scales is None:
        kvq.kvq_absmax_scales_fp8(xs, ss, batch, N, D)
        s_ref = oracle.compute_scales_q(x, 448).reshape(batch, D)
        assert_bits_equal(ss.cpu().numpy().reshape(batch, D), s_ref, "fp8 scales")
    else:
        s_ref = np.ascontiguousarray(given_scales, dtype=np.float32).reshape(batch, D)
        ss.copy_(torch.from_numpy(s_ref.reshape(-1)))
    kvq.kvq_quantize_fp8(xs, ss, cs, batch, N, D)
    q_ref = oracle.quantize_fp8(x, s_ref)
    assert_bits_equal(cs.cpu().numpy().reshape(x.shape), q_ref, "E4M3 codes")
    kvq.kvq_dequantize_fp8(cs, ss, hs, batch, N, D)
    assert_bits_equal(hs.cpu().numpy().reshape(x.shape), oracle.dequantize_fp8(q_ref, s_ref), "fp8 x_hat")
    torch.cuda.synchronize()
    assert bool((dc[:offset] == 0x5A).all() and (dc[offset + n:] == 0x5A).all())
    assert bool((dh[:offset] == 777.0).all() and (dh[offset + n:] == 777.0).all())
    assert bool((ds[:offset] == -5.0).all() and (ds[offset + batch * D:] == -5.0).all())
    return q_ref


@pytest.mark.parametrize("shape", SHAPES + [(1, 1024, 64), (8, 515, 128)], ids=lambda s: "x".join(map(str, s)))
def test_fp8_ragged_shapes(shape):
    rng = np.random.default_rng(seed_of(shape))
    q = fp8_round_trip(make_matrix(rng, *shape))
    assert ((q & 0x7F) != 0x7F).all()                       # no NaN patterns


@pytest.mark.parametrize("offset", [1, 2, 3, 4, 8])
def test_fp8_unaligned_base_pointers(offset):
    rng = np.random.default_rng(offset)
    fp8_round_trip(make_matrix(rng, 2, 70, 64), offset=offset)


def test_fp8_encode_on_a_dense_grid_of_quotients_and_decode_of_every_code():
    """Scale 1 makes the quotient the input itself: every fp32 pattern with 12 low zero bits in the
    range of interest, the neighbourhoods of all rounding boundaries, huge, tiny, subnormal and zero."""
    pats = (np.arange(1 << 20, dtype=np.uint64) << np.uint64(12)).astype(np.uint32)
    y = pats.view(np.float32)
    y = y[np.isfinite(y)]
    vals = oracle.fp8_decode(np.arange(0x7F, dtype=np.uint8)).astype(np.float64)
    mids = ((vals[:-1] + vals[1:]) / 2).astype(np.float32)
    near = np.concatenate([(mids.view(np.uint32).astype(np.int64) + k).astype(np.uint32) for k in range(-3, 4)]).view(np.float32)
    extra = np.array([448.0, 464.0, 463.99, 480.0, 3e38, 1e-45, 2.0 ** -10, 2.0 ** -9, 2.0 ** -126, 0.0],
                     dtype=np.float32)
    y = np.concatenate([y, near, -near, vals[1:].astype(np.float32), extra, -extra])
    D = 64
    y = y[:y.size // D * D].reshape(-1, D)
    fp8_round_trip(y, given_scales=np.ones(D, dtype=np.float32))
    # every finite code through dequantize, with assorted scales (zero, negative, tiny, huge)
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F] * 16 + [0] * 32, dtype=np.uint8)
    codes = codes[:codes.size // D * D].reshape(-1, D)
    s = np.exp(np.random.default_rng(2).uniform(-20, 20, D)).astype(np.float32)
    s[0], s[1], s[2], s[3] = 0.0, -0.25, 2.0 ** -140, 2.0 ** 118
    dcodes = torch.from_numpy(codes).cuda()
    dsc = torch.from_numpy(s).cuda()
    out = torch.empty(codes.shape, dtype=torch.float32, device="cuda")
    kvq.kvq_dequantize_fp8(dcodes, dsc, out, 1, codes.shape[0], D)
    assert_bits_equal(out.cpu().numpy(), oracle.dequantize_fp8(codes, s), "fp8 decode of every code")


def test_fp8_special_scales_and_configs():
    rng = np.random.default_rng(29)
    N, D = 2048, 64
    s = np.exp(rng.uniform(-3, 3, D)).astype(np.float32)
    s[0], s[1], s[2], s[3], s[4], s[5] = 2.0 ** -140, 2.0 ** 120, 1e-3, 3.0, 0.0, -0.25
    x = (rng.standard_normal((N, D)) * np.clip(s, -1e30, 1e30) * 100).astype(np.float32)
    x[:, 0] = (rng.integers(-200, 200, N) * 2.0 ** -141).astype(np.float32)
    x[:, 1] = (rng.standard_normal(N) * 2.0 ** 125).astype(np.float32)
    x[::7, 4] = -0.0
    fp8_round_trip(x, given_scales=s)
    q = fp8_round_trip(W.generate(2)[0])
    assert len(np.unique(q)) > 200
    fp8_round_trip(W.generate(3, slabs=(0, 24)))


def test_matrix_core_scores_do_not_depend_on_the_launch_shape():
    """Integer accumulation: the same slab gives the same bits whether it is scored alone or as one slab of a
    larger batch (different token chunking per workgroup), and from run to run."""
    rng = np.random.default_rng(91)
    N, D, Q = 5000, 128, 8
    x = make_matrix(rng, 3, N, D)
    s = oracle.compute_scales(x)
    codes = torch.from_numpy(oracle.quantize(x, s)).cuda()
    scales = torch.from_numpy(s).cuda()
    qs = torch.from_numpy(rng.standard_normal((3, Q, D)).astype(np.float32)).cuda()
    out_all = torch.empty(3 * Q * N, dtype=torch.float32, device="cuda")
    kvq.kvq_scores_from_codes(qs, Q, codes, scales, 3, N, D, out_all)
    again = torch.empty_like(out_all)
    kvq.kvq_scores_from_codes(qs, Q, codes, scales, 3, N, D, again)
    assert torch.equal(out_all, again)
    for b in range(3):
        alone = torch.empty(Q * N, dtype=torch.float32, device="cuda")
        kvq.kvq_scores_from_codes(qs[b].contiguous(), Q, codes[b].contiguous(), scales[b].contiguous(), 1, N, D, alone)
        assert torch.equal(alone, out_all[b * Q * N:(b + 1) * Q * N])


# ------------------------------------------------------------------ scores from a 4-bit cache
@pytest.mark.parametrize("shape,Q,offset", [((6, 1000, 128), 8, 0), ((1, 4096, 128), 1, 0), ((3, 257, 256), 5, 0),
                                            ((2, 100, 1024), 3, 0), ((1, 300, 64), 4, 0), ((1, 70, 20), 2, 0),
                                            ((2, 515, 128), 16, 0), ((1, 333, 512), 13, 0), ((2, 64, 128), 7, 8),
                                            ((3, 1, 128), 8, 0), ((1, 50, 2048), 3, 0)],
                         ids=lambda v: "x".join(map(str, v)) if isinstance(v, tuple) else str(v))
def test_scores_from_a_four_bit_cache(shape, Q, offset):
    batch, N, D = shape
    rng = np.random.default_rng(N + D + Q)
    x = make_matrix(rng, batch, N, D)
    qs = rng.standard_normal((batch, Q, D)).astype(np.float32)
    qs[:, 0] *= 1e-3
    s_ref = oracle.compute_scales_q(x, 7).reshape(batch, D)
    q_ref = oracle.quantize_q(x, s_ref, 7)
    packed_np = oracle.pack_int4(q_ref)
    buf = torch.zeros(packed_np.size + 64, dtype=torch.uint8, device="cuda")
    packed = buf[offset:offset + packed_np.size]
    packed.copy_(torch.from_numpy(packed_np.reshape(-1)))
    scales = torch.from_numpy(s_ref).cuda()
    out = torch.full((batch * Q * N + 8,), 555.0, dtype=torch.float32, device="cuda")
    kvq.kvq_scores_from_codes_int4(torch.from_numpy(qs).cuda(), Q, packed, scales, batch, N, D, out)
    got = out[:batch * Q * N].cpu().numpy().reshape(batch, Q, N).astype(np.float64)
    assert bool((out[batch * Q * N:] == 555.0).all())
    matrix_cores = D % 128 == 0 and D <= 1024 and offset % 16 == 0
    for b in range(batch):
        ref = oracle.scores_from_codes(qs[b], q_ref[b], s_ref[b])
        xh = oracle.dequantize(q_ref[b], s_ref[b]).astype(np.float64)
        mag = np.abs(qs[b].astype(np.float64)) @ np.abs(xh).T
        if matrix_cores:
            top = np.abs(qs[b].astype(np.float64) * s_ref[b].astype(np.float64)).max(axis=1) * (1 + 2.0 ** -23)
            bound = 2.0 ** -27 * top[:, None] * np.abs(q_ref[b].astype(np.float64)).sum(axis=1)[None, :] \
                + 4 * 2.0 ** -24 * mag
        else:
            bound = scores_bound(D, False) * mag
        bound = bound + (127 * D + 1) * 2.0 ** -150
        err = np.abs(got[b] - ref)
        assert (err <= bound).all(), (b, float((err / bound).max()))


def test_scores_int4_rejects_an_odd_channel_count():
    z = torch.zeros(64, dtype=torch.float32, device="cuda")
    p = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(kvq.KvqError) as e:
        kvq.kvq_scores_from_codes_int4(z, 1, p, z, 1, 3, 5, z)
    assert e.value.status == kvq.ERR_ARG
