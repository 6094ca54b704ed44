"""ctypes binding of libkvq.so: same names as include/kvq.h and include/kvq_bench.h, argument marshalling only.

Arguments may be torch tensors (anything with .data_ptr()), or raw integer
device addresses.  `stream` is a raw hipStream_t value (for torch:
torch.cuda.current_stream().cuda_stream) or None for torch's current stream
when torch is importable and a GPU is present, else the default stream.

There is no CPU fallback: if the shared library is missing, loading raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvq.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_OVERFLOW, ERR_HIP, ERR_ARG, ERR_LIMIT = -1, -2, -3, -4, -5, -6
STATIC_SCRATCH_FLOATS = 2097152
OPT_CODEC_WIDTH, OPT_CODEC_UNROLL, OPT_BLOCKS_PER_CU, OPT_NONTEMPORAL = 1, 2, 3, 4
OPT_BLOCK_THREADS, OPT_PASSES_PER_BLOCK, OPT_ABSMAX_UNROLL, OPT_ABSMAX_PASSES, OPT_ABSMAX_SPAN = 6, 7, 8, 9, 10
OPT_ABSMAX_BLOCKS_PER_CU = 11
OPT_APPEND_BLOCKS_PER_CU = 12
OPT_FUSED_MIN_LANES = 13
OPT_FUSED_MAX_ROWS = 14
OPT_ATTN_FORM = 15
OPT_FUSED_TALL = 16

# the method and its workspace calls: include/kvq.h
EXPORTS = (
    "kvq_absmax_scales", "kvq_absmax_scales_static", "kvq_quantize", "kvq_dequantize", "kvq_quantize_fused",
    "kvq_absmax_scales_t", "kvq_quantize_t", "kvq_dequantize_t",
    "kvq_absmax_scales_int4", "kvq_quantize_int4", "kvq_dequantize_int4",
    "kvq_absmax_scales_fp8", "kvq_quantize_fp8", "kvq_dequantize_fp8",
    "kvq_append", "kvq_append_t", "kvq_append_int4",
    "kvq_roundtrip_error", "kvq_attn_score_error", "kvq_scores_from_codes", "kvq_scores_from_codes_int4",
    "kvq_prepare_stream", "kvq_release_stream", "kvq_status_string", "kvq_last_hip_error",
)
# measurement and ablation: include/kvq_bench.h
BENCH_EXPORTS = (
    "kvq_quantize_variant", "kvq_probe_stream", "kvq_probe_clock", "kvq_plan", "kvq_set_option", "kvq_get_option",
)

_lib = None


class KvqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().kvq_status_string(status).decode()
        if status == ERR_HIP:
            msg += " (hipError_t %d)" % lib().kvq_last_hip_error()
        super().__init__("%s: %s" % (where, msg))


def lib():
    """The loaded shared library (raises OSError with a build hint when it is absent)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("%s not found: build it with `python -m paper_2601_04719_amd.build` "
                          "(there is no CPU fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        p, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
        L.kvq_absmax_scales.argtypes = [p, p, i64, i64, i64, p]
        L.kvq_absmax_scales_static.argtypes = [p, p, i64, i64, i64, p]
        L.kvq_absmax_scales_static.restype = i32
        L.kvq_quantize.argtypes = [p, p, p, i64, i64, i64, p]
        L.kvq_dequantize.argtypes = [p, p, p, i64, i64, i64, p]
        L.kvq_quantize_fused.argtypes = [p, p, p, i64, i64, i64, p]
        L.kvq_absmax_scales_t.argtypes = [i32, p, p, i64, i64, i64, p]
        L.kvq_quantize_t.argtypes = [i32, p, p, p, i64, i64, i64, p]
        L.kvq_dequantize_t.argtypes = [i32, p, p, p, i64, i64, i64, p]
        for name in ("kvq_absmax_scales_t", "kvq_quantize_t", "kvq_dequantize_t"):
            getattr(L, name).restype = i32
        L.kvq_absmax_scales_int4.argtypes = [p, p, i64, i64, i64, p]
        L.kvq_quantize_int4.argtypes = [p, p, p, i64, i64, i64, p]
        L.kvq_dequantize_int4.argtypes = [p, p, p, i64, i64, i64, p]
        for name in ("kvq_absmax_scales_int4", "kvq_quantize_int4", "kvq_dequantize_int4"):
            getattr(L, name).restype = i32
        L.kvq_absmax_scales_fp8.argtypes = [p, p, i64, i64, i64, p]
        L.kvq_quantize_fp8.argtypes = [p, p, p, i64, i64, i64, p]
        L.kvq_dequantize_fp8.argtypes = [p, p, p, i64, i64, i64, p]
        for name in ("kvq_absmax_scales_fp8", "kvq_quantize_fp8", "kvq_dequantize_fp8"):
            getattr(L, name).restype = i32
        L.kvq_append.argtypes = [p, p, p, p, i64, i64, i64, i64, i64, p]
        L.kvq_append.restype = i32
        L.kvq_append_t.argtypes = [i32, p, p, p, p, i64, i64, i64, i64, i64, p]
        L.kvq_append_t.restype = i32
        L.kvq_append_int4.argtypes = [p, p, p, p, i64, i64, i64, i64, i64, p]
        L.kvq_append_int4.restype = i32
        L.kvq_plan.argtypes = [i32, i64, i64, i64, i32, i32, p]
        L.kvq_plan.restype = i32
        L.kvq_prepare_stream.argtypes = [p]
        L.kvq_prepare_stream.restype = i32
        L.kvq_release_stream.argtypes = [p]
        L.kvq_release_stream.restype = i32
        L.kvq_quantize_variant.argtypes = [i32, p, p, p, i64, i64, i64, p]
        L.kvq_quantize_variant.restype = i32
        L.kvq_scores_from_codes.argtypes = [p, i64, p, p, i64, i64, i64, p, p]
        L.kvq_scores_from_codes.restype = i32
        L.kvq_scores_from_codes_int4.argtypes = [p, i64, p, p, i64, i64, i64, p, p]
        L.kvq_scores_from_codes_int4.restype = i32
        L.kvq_probe_stream.argtypes = [i32, p, p, p, p, p, i64, i64, i64, p]
        L.kvq_probe_stream.restype = i32
        L.kvq_probe_clock.argtypes = [p, i32, p]
        L.kvq_probe_clock.restype = i32
        L.kvq_roundtrip_error.argtypes = [p, p, p, p, i64, i64, i64, p, p, p]
        L.kvq_attn_score_error.argtypes = [p, i64, p, p, p, p, i64, i64, p, p]
        for name in ("kvq_absmax_scales", "kvq_quantize", "kvq_dequantize", "kvq_quantize_fused",
                     "kvq_roundtrip_error", "kvq_attn_score_error"):
            getattr(L, name).restype = i32
        L.kvq_status_string.argtypes = [i32]
        L.kvq_status_string.restype = ctypes.c_char_p
        L.kvq_last_hip_error.argtypes = []
        L.kvq_last_hip_error.restype = i32
        L.kvq_set_option.argtypes = [i32, i32]
        L.kvq_set_option.restype = i32
        L.kvq_get_option.argtypes = [i32]
        L.kvq_get_option.restype = i32
        _lib = L
    return _lib


def _addr(a):
    if a is None:
        return None
    if isinstance(a, int):
        return a
    return a.data_ptr()


def _stream(stream):
    if stream is not None:
        return stream
    try:
        import torch
        if torch.cuda.is_available():
            return torch.cuda.current_stream().cuda_stream
    except ImportError:
        pass
    return None


def _check(status, where):
    if status != OK:
        raise KvqError(status, where)


def kvq_absmax_scales(x, scales, batch, N, D, stream=None):
    _check(lib().kvq_absmax_scales(_addr(x), _addr(scales), batch, N, D, _stream(stream)), "kvq_absmax_scales")


def kvq_absmax_scales_static(x, scales, batch, N, D, stream=None):
    _check(lib().kvq_absmax_scales_static(_addr(x), _addr(scales), batch, N, D, _stream(stream)),
           "kvq_absmax_scales_static")


def kvq_quantize(x, scales, codes, batch, N, D, stream=None):
    _check(lib().kvq_quantize(_addr(x), _addr(scales), _addr(codes), batch, N, D, _stream(stream)), "kvq_quantize")


def kvq_dequantize(codes, scales, x_hat, batch, N, D, stream=None):
    _check(lib().kvq_dequantize(_addr(codes), _addr(scales), _addr(x_hat), batch, N, D, _stream(stream)),
           "kvq_dequantize")


def kvq_quantize_fused(x, scales, codes, batch, N, D, stream=None):
    _check(lib().kvq_quantize_fused(_addr(x), _addr(scales), _addr(codes), batch, N, D, _stream(stream)),
           "kvq_quantize_fused")


DTYPE_F32, DTYPE_F16, DTYPE_BF16 = 0, 1, 2


def kvq_absmax_scales_t(dtype, x, scales, batch, N, D, stream=None):
    _check(lib().kvq_absmax_scales_t(dtype, _addr(x), _addr(scales), batch, N, D, _stream(stream)),
           "kvq_absmax_scales_t")


def kvq_quantize_t(dtype, x, scales, codes, batch, N, D, stream=None):
    _check(lib().kvq_quantize_t(dtype, _addr(x), _addr(scales), _addr(codes), batch, N, D, _stream(stream)),
           "kvq_quantize_t")


def kvq_dequantize_t(dtype, codes, scales, x_hat, batch, N, D, stream=None):
    _check(lib().kvq_dequantize_t(dtype, _addr(codes), _addr(scales), _addr(x_hat), batch, N, D, _stream(stream)),
           "kvq_dequantize_t")


def kvq_absmax_scales_int4(x, scales, batch, N, D, stream=None):
    _check(lib().kvq_absmax_scales_int4(_addr(x), _addr(scales), batch, N, D, _stream(stream)),
           "kvq_absmax_scales_int4")


def kvq_quantize_int4(x, scales, packed, batch, N, D, stream=None):
    _check(lib().kvq_quantize_int4(_addr(x), _addr(scales), _addr(packed), batch, N, D, _stream(stream)),
           "kvq_quantize_int4")


def kvq_dequantize_int4(packed, scales, x_hat, batch, N, D, stream=None):
    _check(lib().kvq_dequantize_int4(_addr(packed), _addr(scales), _addr(x_hat), batch, N, D, _stream(stream)),
           "kvq_dequantize_int4")


def kvq_absmax_scales_fp8(x, scales, batch, N, D, stream=None):
    _check(lib().kvq_absmax_scales_fp8(_addr(x), _addr(scales), batch, N, D, _stream(stream)),
           "kvq_absmax_scales_fp8")


def kvq_quantize_fp8(x, scales, codes, batch, N, D, stream=None):
    _check(lib().kvq_quantize_fp8(_addr(x), _addr(scales), _addr(codes), batch, N, D, _stream(stream)),
           "kvq_quantize_fp8")


def kvq_dequantize_fp8(codes, scales, x_hat, batch, N, D, stream=None):
    _check(lib().kvq_dequantize_fp8(_addr(codes), _addr(scales), _addr(x_hat), batch, N, D, _stream(stream)),
           "kvq_dequantize_fp8")


def kvq_append(x_new, scales, scales_prev, codes, batch, n_old, m, capacity, D, stream=None):
    _check(lib().kvq_append(_addr(x_new), _addr(scales), _addr(scales_prev), _addr(codes), batch, n_old, m,
                            capacity, D, _stream(stream)), "kvq_append")


def kvq_append_int4(x_new, scales, scales_prev, packed, batch, n_old, m, capacity, D, stream=None):
    _check(lib().kvq_append_int4(_addr(x_new), _addr(scales), _addr(scales_prev), _addr(packed), batch, n_old, m,
                                 capacity, D, _stream(stream)), "kvq_append_int4")


def kvq_append_t(dtype, x_new, scales, scales_prev, codes, batch, n_old, m, capacity, D, stream=None):
    _check(lib().kvq_append_t(dtype, _addr(x_new), _addr(scales), _addr(scales_prev), _addr(codes), batch, n_old, m,
                              capacity, D, _stream(stream)), "kvq_append_t")


def kvq_prepare_stream(stream=None):
    _check(lib().kvq_prepare_stream(_stream(stream)), "kvq_prepare_stream")


def kvq_release_stream(stream=None):
    _check(lib().kvq_release_stream(_stream(stream)), "kvq_release_stream")


PLAN_ABSMAX, PLAN_QUANTIZE, PLAN_DEQUANTIZE = 0, 1, 2
PLAN_FIELDS = ("V", "J", "block", "TX", "ctiles", "rchunks", "rows_per_chunk", "unroll")


def kvq_plan(call, batch, N, D, vector_access=True, compute_units=256):
    """Host-side launch plan as a dict (see include/kvq.h); no device is touched."""
    out = (ctypes.c_int64 * 8)()
    _check(lib().kvq_plan(call, batch, N, D, int(bool(vector_access)), compute_units,
                          ctypes.cast(out, ctypes.c_void_p)), "kvq_plan")
    return dict(zip(PLAN_FIELDS, (int(v) for v in out)))


VARIANT_PRODUCTION, VARIANT_NAIVE, VARIANT_TILED, VARIANT_COARSENED, VARIANT_VECTORIZED = 0, 1, 2, 3, 4
VARIANT_NAMES = {0: "production", 1: "naive", 2: "tiled", 3: "coarsened", 4: "vectorized"}


def kvq_quantize_variant(variant, x, scales, codes, batch, N, D, stream=None):
    _check(lib().kvq_quantize_variant(variant, _addr(x), _addr(scales), _addr(codes), batch, N, D, _stream(stream)),
           "kvq_quantize_variant")


def kvq_roundtrip_error(x, x_hat, codes, scales, batch, N, D, sumsq_out, maxabs_out, stream=None):
    _check(lib().kvq_roundtrip_error(_addr(x), _addr(x_hat), _addr(codes), _addr(scales), batch, N, D,
                                     _addr(sumsq_out), _addr(maxabs_out), _stream(stream)), "kvq_roundtrip_error")


def kvq_attn_score_error(queries, Q, k, k_hat, codes, scales, N, D, mean_abs_out, stream=None):
    _check(lib().kvq_attn_score_error(_addr(queries), Q, _addr(k), _addr(k_hat), _addr(codes), _addr(scales),
                                      N, D, _addr(mean_abs_out), _stream(stream)), "kvq_attn_score_error")


def kvq_scores_from_codes(queries, Q, codes, scales, batch, N, D, scores_out, stream=None):
    _check(lib().kvq_scores_from_codes(_addr(queries), Q, _addr(codes), _addr(scales), batch, N, D,
                                       _addr(scores_out), _stream(stream)), "kvq_scores_from_codes")


def kvq_scores_from_codes_int4(queries, Q, packed, scales, batch, N, D, scores_out, stream=None):
    _check(lib().kvq_scores_from_codes_int4(_addr(queries), Q, _addr(packed), _addr(scales), batch, N, D,
                                            _addr(scores_out), _stream(stream)), "kvq_scores_from_codes_int4")


def kvq_probe_stream(mode, src_f32, dst_f32, src_i8, dst_i8, scales, batch, N, D, stream=None):
    _check(lib().kvq_probe_stream(mode, _addr(src_f32), _addr(dst_f32), _addr(src_i8), _addr(dst_i8), _addr(scales),
                                  batch, N, D, _stream(stream)), "kvq_probe_stream")


def kvq_probe_clock(ticks_out, microseconds, stream=None):
    _check(lib().kvq_probe_clock(_addr(ticks_out), microseconds, _stream(stream)), "kvq_probe_clock")


def kvq_status_string(status):
    return lib().kvq_status_string(status).decode()


def kvq_last_hip_error():
    return lib().kvq_last_hip_error()


def kvq_set_option(key, value):
    _check(lib().kvq_set_option(key, value), "kvq_set_option")


def kvq_get_option(key):
    return lib().kvq_get_option(key)
