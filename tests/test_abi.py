"""The C-ABI library loads, exports every symbol include/kvq.h declares, and rejects bad
arguments on the host before any HIP call.  CPU only (no kernel is launched)."""
import ctypes
import os
import re

import pytest

from paper_2601_04719_amd import kvq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "kvq.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvq_[a-z_0-9]+)\s*\(", text)))


def test_header_and_binding_list_the_same_entry_points():
    names = declared_functions()
    assert {"kvq_absmax_scales", "kvq_quantize", "kvq_dequantize", "kvq_roundtrip_error",
            "kvq_attn_score_error"} <= set(names)
    assert sorted(kvq.EXPORTS) == names
    for n in names:
        assert callable(getattr(kvq, n)), n


def test_library_exports_every_declared_symbol():
    L = kvq.lib()
    for n in declared_functions():
        assert getattr(L, n) is not None


def test_status_strings():
    assert kvq.kvq_status_string(0) == "KVQ_OK"
    for s in (-1, -2, -3, -4, -5):
        assert kvq.kvq_status_string(s).startswith("KVQ_ERR_")
    assert "unknown" in kvq.kvq_status_string(-99)


def test_argument_errors_are_reported_before_any_launch():
    L = kvq.lib()
    fake = 0x1000   # never dereferenced: every call below must fail validation first
    assert L.kvq_absmax_scales(None, fake, 1, 4, 4, None) == kvq.ERR_NULL
    assert L.kvq_absmax_scales(fake, None, 1, 4, 4, None) == kvq.ERR_NULL
    assert L.kvq_quantize(fake, fake, None, 1, 4, 4, None) == kvq.ERR_NULL
    assert L.kvq_dequantize(None, fake, fake, 1, 4, 4, None) == kvq.ERR_NULL
    assert L.kvq_quantize_fused(fake, None, fake, 1, 4, 4, None) == kvq.ERR_NULL
    for bad in [(0, 4, 4), (1, 0, 4), (1, 4, 0), (-1, 4, 4), (1, -4, 4)]:
        assert L.kvq_absmax_scales(fake, fake, *bad, None) == kvq.ERR_SHAPE
        assert L.kvq_quantize(fake, fake, fake, *bad, None) == kvq.ERR_SHAPE
        assert L.kvq_dequantize(fake, fake, fake, *bad, None) == kvq.ERR_SHAPE
        assert L.kvq_roundtrip_error(fake, fake, None, None, *bad, fake, fake, None) == kvq.ERR_SHAPE
    big = 1 << 40
    assert L.kvq_quantize(fake, fake, fake, 1, big, big, None) == kvq.ERR_OVERFLOW
    assert L.kvq_quantize(fake, fake, fake, big, big, 2, None) == kvq.ERR_OVERFLOW
    # round-trip error: either x_hat or (codes and scales)
    assert L.kvq_roundtrip_error(fake, None, None, fake, 1, 4, 4, fake, fake, None) == kvq.ERR_NULL
    assert L.kvq_roundtrip_error(fake, None, fake, None, 1, 4, 4, fake, fake, None) == kvq.ERR_NULL
    assert L.kvq_roundtrip_error(fake, fake, None, None, 1, 4, 4, None, fake, None) == kvq.ERR_NULL
    assert L.kvq_roundtrip_error(fake, fake, None, None, 1, 4, 4, fake + 4, fake, None) == kvq.ERR_ARG
    assert L.kvq_attn_score_error(fake, 0, fake, fake, None, None, 4, 4, fake, None) == kvq.ERR_SHAPE
    assert L.kvq_attn_score_error(fake, 2, fake, None, None, None, 4, 4, fake, None) == kvq.ERR_NULL
    assert L.kvq_attn_score_error(None, 2, fake, fake, None, None, 4, 4, fake, None) == kvq.ERR_NULL
    with pytest.raises(kvq.KvqError) as e:
        kvq.kvq_quantize(fake, fake, fake, 1, 0, 4)
    assert e.value.status == kvq.ERR_SHAPE and "KVQ_ERR_SHAPE" in str(e.value)


def test_options_round_trip_and_reject_bad_values():
    for key, good, bad in [(kvq.OPT_CODEC_WIDTH, 8, 3), (kvq.OPT_CODEC_UNROLL, 4, 3),
                           (kvq.OPT_BLOCKS_PER_CU, 16, 0), (kvq.OPT_NONTEMPORAL, 0, 2),
                           (kvq.OPT_BLOCK_THREADS, 128, 100), (kvq.OPT_PASSES_PER_BLOCK, 0, -1),
                           (kvq.OPT_ABSMAX_UNROLL, 4, 5), (kvq.OPT_ABSMAX_PASSES, 2, -1),
                           (kvq.OPT_ABSMAX_SPAN, 2, 3), (kvq.OPT_ABSMAX_BLOCKS_PER_CU, 4, 0),
                           (kvq.OPT_APPEND_BLOCKS_PER_CU, 32, 0)]:
        old = kvq.kvq_get_option(key)
        kvq.kvq_set_option(key, good)
        assert kvq.kvq_get_option(key) == good
        with pytest.raises(kvq.KvqError):
            kvq.kvq_set_option(key, bad)
        assert kvq.kvq_get_option(key) == good
        kvq.kvq_set_option(key, old)
    with pytest.raises(kvq.KvqError):
        kvq.kvq_set_option(99, 1)


def test_oracle_and_product_share_no_code():
    """Neither side imports, includes or links the other."""
    for dirpath, _, files in os.walk(os.path.join(ROOT, "paper_2601_04719_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"import\s+oracle|from\s+oracle|oracle/|kvq_oracle", src), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            src = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2601_04719_amd" not in src and "libkvq.so" not in src and "hip/" not in src, f
