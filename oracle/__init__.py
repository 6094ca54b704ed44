"""numpy front end of the CPU oracle (oracle/kvq_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import this package.  It holds no code of the
HIP library and the HIP library holds none of it.

All arrays are C-contiguous numpy arrays; a matrix is [N, D] (tokens x
channels) or [batch, N, D]; scales are [D] or [batch, D].
"""
import ctypes
import threading

import numpy as np

from . import build as _build

_lib = None
_lock = threading.Lock()

_i64 = ctypes.c_int64
_fp = ctypes.POINTER(ctypes.c_float)
_bp = ctypes.POINTER(ctypes.c_int8)
_dp = ctypes.POINTER(ctypes.c_double)


def lib():
    """Load (building first if the source is newer) the oracle shared library."""
    global _lib
    with _lock:
        if _lib is None:
            path = _build.build(force=False)
            L = ctypes.CDLL(path)
            L.kvq_oracle_compute_scales.argtypes = [_fp, _fp, _i64, _i64, _i64]
            L.kvq_oracle_compute_scales.restype = None
            L.kvq_oracle_quantize.argtypes = [_fp, _fp, _bp, _i64, _i64, _i64]
            L.kvq_oracle_quantize.restype = None
            L.kvq_oracle_dequantize.argtypes = [_bp, _fp, _fp, _i64, _i64, _i64]
            L.kvq_oracle_dequantize.restype = None
            L.kvq_oracle_roundtrip_error.argtypes = [_fp, _fp, _i64, _dp, _fp]
            L.kvq_oracle_roundtrip_error.restype = None
            L.kvq_oracle_attn_score_error.argtypes = [_fp, _i64, _fp, _fp, _i64, _i64, _dp]
            L.kvq_oracle_attn_score_error.restype = None
            L.kvq_oracle_scores_from_codes.argtypes = [_fp, _i64, _bp, _fp, _i64, _i64, _dp]
            L.kvq_oracle_scores_from_codes.restype = None
            L.kvq_oracle_compute_scales_q.argtypes = [_fp, _fp, _i64, _i64, _i64, ctypes.c_int]
            L.kvq_oracle_compute_scales_q.restype = None
            L.kvq_oracle_quantize_q.argtypes = [_fp, _fp, _bp, _i64, _i64, _i64, ctypes.c_int]
            L.kvq_oracle_quantize_q.restype = None
            _u8 = ctypes.POINTER(ctypes.c_uint8)
            L.kvq_oracle_fp8_encode.argtypes = [_fp, _u8, _i64]
            L.kvq_oracle_fp8_encode.restype = None
            L.kvq_oracle_fp8_decode.argtypes = [_u8, _fp, _i64]
            L.kvq_oracle_fp8_decode.restype = None
            L.kvq_oracle_quantize_fp8.argtypes = [_fp, _fp, _u8, _i64, _i64, _i64]
            L.kvq_oracle_quantize_fp8.restype = None
            L.kvq_oracle_dequantize_fp8.argtypes = [_u8, _fp, _fp, _i64, _i64, _i64]
            L.kvq_oracle_dequantize_fp8.restype = None
            _lib = L
    return _lib


def _shape3(a):
    if a.ndim == 2:
        return 1, a.shape[0], a.shape[1]
    if a.ndim == 3:
        return a.shape
    raise ValueError("expected [N, D] or [batch, N, D], got shape %r" % (a.shape,))


def _f32(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("expected float32, got %s" % a.dtype)
    return a


def _ptr(a, t):
    return a.ctypes.data_as(t)


def compute_scales(x):
    """scales[b, d] = max_t |x[b, t, d]| / 127 (fp32)."""
    x = _f32(x)
    b, n, d = _shape3(x)
    out = np.empty((b, d), dtype=np.float32)
    lib().kvq_oracle_compute_scales(_ptr(x, _fp), _ptr(out, _fp), b, n, d)
    return out if x.ndim == 3 else out[0]


def quantize(x, scales):
    """codes = clamp(rint(x / scale), -127, 127) as int8; 0 where scale == 0."""
    x = _f32(x)
    scales = _f32(scales)
    b, n, d = _shape3(x)
    if scales.size != b * d:
        raise ValueError("scales must hold batch*D values")
    out = np.empty(x.shape, dtype=np.int8)
    lib().kvq_oracle_quantize(_ptr(x, _fp), _ptr(scales, _fp), _ptr(out, _bp), b, n, d)
    return out


def dequantize(codes, scales):
    """x_hat = float(code) * scale (fp32)."""
    codes = np.ascontiguousarray(codes)
    if codes.dtype != np.int8:
        raise TypeError("expected int8 codes")
    scales = _f32(scales)
    b, n, d = _shape3(codes)
    if scales.size != b * d:
        raise ValueError("scales must hold batch*D values")
    out = np.empty(codes.shape, dtype=np.float32)
    lib().kvq_oracle_dequantize(_ptr(codes, _bp), _ptr(scales, _fp), _ptr(out, _fp), b, n, d)
    return out


def roundtrip_error(x, x_hat):
    """Returns (sumsq: float64, maxabs: float32) of x - x_hat over all elements."""
    x = _f32(x)
    x_hat = _f32(x_hat)
    if x.shape != x_hat.shape:
        raise ValueError("shape mismatch")
    s = ctypes.c_double(0.0)
    m = ctypes.c_float(0.0)
    lib().kvq_oracle_roundtrip_error(_ptr(x, _fp), _ptr(x_hat, _fp), x.size,
                                     ctypes.byref(s), ctypes.byref(m))
    return float(s.value), np.float32(m.value)


def attn_score_error(queries, k, k_hat):
    """mean over (query j, token t) of |q_j . k_t - q_j . k_hat_t| (fp64)."""
    queries = _f32(queries)
    k = _f32(k)
    k_hat = _f32(k_hat)
    if k.ndim != 2 or k.shape != k_hat.shape or queries.ndim != 2 or queries.shape[1] != k.shape[1]:
        raise ValueError("expected queries [Q, D], k and k_hat [N, D]")
    r = ctypes.c_double(0.0)
    lib().kvq_oracle_attn_score_error(_ptr(queries, _fp), queries.shape[0], _ptr(k, _fp),
                                      _ptr(k_hat, _fp), k.shape[0], k.shape[1], ctypes.byref(r))
    return float(r.value)


def scores_from_codes(queries, codes, scales):
    """out[j, t] = q_j . k_hat_t with k_hat = float(code) * scale (fp32), dot product in fp64; [Q, N] float64."""
    queries = _f32(queries)
    scales = _f32(scales)
    codes = np.ascontiguousarray(codes)
    if codes.dtype != np.int8 or codes.ndim != 2 or queries.ndim != 2 or queries.shape[1] != codes.shape[1] \
            or scales.size != codes.shape[1]:
        raise ValueError("expected queries [Q, D] float32, codes [N, D] int8, scales [D] float32")
    out = np.empty((queries.shape[0], codes.shape[0]), dtype=np.float64)
    lib().kvq_oracle_scores_from_codes(_ptr(queries, _fp), queries.shape[0], _ptr(codes, _bp), _ptr(scales, _fp),
                                       codes.shape[0], codes.shape[1], _ptr(out, _dp))
    return out


# ---------------------------------------------------------------------------------------------
# 16-bit matrices ("Memory Bottleneck in LLM Inference": caches are kept in FP16-class formats).
# A 16-bit value widens to fp32 exactly, so scales and codes of a 16-bit matrix are those of the
# widened matrix; dequantization rounds the fp32 product once more, to nearest even.
# ---------------------------------------------------------------------------------------------
def widen16(bits, fmt):
    """uint16 bit patterns of fp16 ('f16') or bfloat16 ('bf16') values -> float32 (exact)."""
    bits = np.ascontiguousarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError("expected uint16 bit patterns")
    if fmt == "f16":
        return bits.view(np.float16).astype(np.float32)
    if fmt == "bf16":
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    raise ValueError(fmt)


def narrow16(x, fmt):
    """float32 -> nearest fp16 / bfloat16 (ties to even), as uint16 bit patterns.  Finite inputs."""
    x = _f32(x)
    if fmt == "f16":
        with np.errstate(over="ignore"):
            return x.astype(np.float16).view(np.uint16)
    if fmt == "bf16":
        u = x.view(np.uint32).astype(np.uint64)
        lsb = (u >> np.uint64(16)) & np.uint64(1)            # parity of the kept part decides a tie
        return ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)).astype(np.uint16)
    raise ValueError(fmt)


def dequantize_as(codes, scales, fmt):
    """x_hat = round_to_16bit(float32(code) * scale): Eq. (dequant_op) in fp32, then one rounding."""
    return narrow16(dequantize(codes, scales), fmt)


# ---------------------------------------------------------------------------------------------
# 4-bit codes (Limitations, "Lower bit-widths"): the same method with the range [-7, 7]
# ---------------------------------------------------------------------------------------------
def compute_scales_q(x, qmax):
    """scales[b, d] = max_t |x[b, t, d]| / qmax (fp32)."""
    x = _f32(x)
    b, n, d = _shape3(x)
    out = np.empty((b, d), dtype=np.float32)
    lib().kvq_oracle_compute_scales_q(_ptr(x, _fp), _ptr(out, _fp), b, n, d, int(qmax))
    return out if x.ndim == 3 else out[0]


def quantize_q(x, scales, qmax):
    """codes = clamp(rint(x / scale), -qmax, qmax), one code per int8; 0 where scale == 0."""
    x = _f32(x)
    scales = _f32(scales)
    b, n, d = _shape3(x)
    if scales.size != b * d:
        raise ValueError("scales must hold batch*D values")
    out = np.empty(x.shape, dtype=np.int8)
    lib().kvq_oracle_quantize_q(_ptr(x, _fp), _ptr(scales, _fp), _ptr(out, _bp), b, n, d, int(qmax))
    return out


def pack_int4(codes):
    """Two 4-bit two's-complement codes per byte: channel 2j in the low nibble, 2j+1 in the high nibble."""
    codes = np.ascontiguousarray(codes)
    if codes.dtype != np.int8 or codes.shape[-1] % 2:
        raise ValueError("expected int8 codes with an even number of channels")
    if codes.min(initial=0) < -8 or codes.max(initial=0) > 7:
        raise ValueError("codes do not fit 4 bits")
    u = codes.view(np.uint8) & np.uint8(0x0F)
    return (u[..., 0::2] | (u[..., 1::2] << np.uint8(4))).astype(np.uint8)


def unpack_int4(packed):
    """Inverse of pack_int4: uint8 [..., D/2] -> int8 [..., D] with sign extension."""
    packed = np.ascontiguousarray(packed)
    if packed.dtype != np.uint8:
        raise TypeError("expected uint8")
    lo = (packed & np.uint8(0x0F)).astype(np.int8)
    hi = (packed >> np.uint8(4)).astype(np.int8)
    lo = np.where(lo > 7, lo - 16, lo).astype(np.int8)
    hi = np.where(hi > 7, hi - 16, hi).astype(np.int8)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


# ---------------------------------------------------------------------------------------------
# Streaming append (Limitations, "Dynamic quantization": scales that adapt during inference;
# Future Work: streaming workloads).  The cache keeps only codes and scales, so when new tokens
# raise a channel's absmax the cached codes of that channel are re-expressed in the new scale
# from their reconstruction:  code' = Q(code * s_old ; s_new), with Q and the product being
# Eq. (quant_op) and Eq. (dequant_op).  Built from the functions above, nothing else.
# ---------------------------------------------------------------------------------------------
def append_q(codes, scales, n_old, x_new, qmax):
    """Streaming append with the integer range [-qmax, qmax] (127: 8-bit codes, 7: 4-bit codes).

    codes [batch, capacity, D] int8 (rows [0, n_old) valid), scales [batch, D], x_new [batch, m, D].
    Returns (codes', scales', scales_prev): rows [0, n_old + m) of codes' valid, the rest untouched."""
    codes = np.ascontiguousarray(codes)
    x_new = _f32(x_new)
    if codes.ndim != 3 or x_new.ndim != 3 or codes.dtype != np.int8:
        raise ValueError("expected codes [batch, capacity, D] int8 and x_new [batch, m, D] float32")
    batch, cap, D = codes.shape
    m = x_new.shape[1]
    s_old = _f32(scales).reshape(batch, D)
    if x_new.shape[0] != batch or x_new.shape[2] != D or not (0 <= n_old and n_old + m <= cap):
        raise ValueError("shape mismatch or capacity exceeded")
    cand = compute_scales_q(x_new, qmax).reshape(batch, D)         # absmax of the new tokens / qmax
    s_new = np.where(cand > s_old, cand, s_old).astype(np.float32)
    grew = s_new > s_old                                           # [batch, D]
    out = codes.copy()
    if n_old:
        cached = np.ascontiguousarray(codes[:, :n_old])
        again = quantize_q(dequantize(cached, s_old), s_new, qmax)  # reconstruction, then the new scale
        out[:, :n_old] = np.where(grew[:, None, :], again, cached)
    out[:, n_old:n_old + m] = quantize_q(x_new, s_new, qmax)
    return out, s_new, s_old.copy()


def append(codes, scales, n_old, x_new):
    """append_q for 8-bit codes."""
    return append_q(codes, scales, n_old, x_new, 127)


# ---------------------------------------------------------------------------------------------
# FP8 codes (Future Work, "GPU-specific numeric formats such as FP8"): OCP E4M3 instead of int8
# ---------------------------------------------------------------------------------------------
_u8p = ctypes.POINTER(ctypes.c_uint8)


def fp8_encode(y):
    """float32 -> E4M3 bit patterns (uint8): round to nearest even, saturate at +-448."""
    y = _f32(y)
    out = np.empty(y.shape, dtype=np.uint8)
    lib().kvq_oracle_fp8_encode(_ptr(y, _fp), _ptr(out, _u8p), y.size)
    return out


def fp8_decode(codes):
    """E4M3 bit patterns (uint8, no NaN patterns) -> float32 (exact)."""
    codes = np.ascontiguousarray(codes)
    if codes.dtype != np.uint8:
        raise TypeError("expected uint8")
    out = np.empty(codes.shape, dtype=np.float32)
    lib().kvq_oracle_fp8_decode(_ptr(codes, _u8p), _ptr(out, _fp), codes.size)
    return out


def quantize_fp8(x, scales):
    """codes = E4M3(x / scale) as uint8; 0 where scale == 0."""
    x = _f32(x)
    scales = _f32(scales)
    b, n, d = _shape3(x)
    if scales.size != b * d:
        raise ValueError("scales must hold batch*D values")
    out = np.empty(x.shape, dtype=np.uint8)
    lib().kvq_oracle_quantize_fp8(_ptr(x, _fp), _ptr(scales, _fp), _ptr(out, _u8p), b, n, d)
    return out


def dequantize_fp8(codes, scales):
    """x_hat = value(code) * scale (fp32)."""
    codes = np.ascontiguousarray(codes)
    if codes.dtype != np.uint8:
        raise TypeError("expected uint8 codes")
    scales = _f32(scales)
    b, n, d = _shape3(codes)
    if scales.size != b * d:
        raise ValueError("scales must hold batch*D values")
    out = np.empty(codes.shape, dtype=np.float32)
    lib().kvq_oracle_dequantize_fp8(_ptr(codes, _u8p), _ptr(scales, _fp), _ptr(out, _fp), b, n, d)
    return out
