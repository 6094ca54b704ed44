"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer.

oracle/kvq_oracle.c is compiled together with oracle/sanitize_driver.c with
-fsanitize=address,undefined -fno-sanitize-recover=all; the driver calls every oracle function on
buffers of exactly the documented sizes.  An access outside a buffer or undefined arithmetic ends the
run with a report.  Its output must equal, byte for byte, what the ordinary build of the oracle
returns for the same inputs (through the numpy front end)."""
import os
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCES = [os.path.join(ROOT, "oracle", "kvq_oracle.c"), os.path.join(ROOT, "oracle", "sanitize_driver.c")]
# the sanitizer runtimes are linked statically, so that they are first whatever else the process loads
SANITIZE = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
            "-static-libasan", "-static-libubsan"]


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("sanitized") / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fno-fast-math", "-ffp-contract=off", "-Wall", "-Wextra"] + SANITIZE
    subprocess.run(cmd + ["-o", exe] + SOURCES + ["-lm"], check=True)
    return exe


def run_driver(exe, tmp_path, x, queries):
    batch, N, D = x.shape
    src, dst = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(src, "wb") as f:
        f.write(np.array([batch, N, D, queries.shape[0]], dtype=np.int64).tobytes())
        f.write(x.tobytes())
        f.write(queries.tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe, src, dst], env=env, capture_output=True, text=True, timeout=300)
    assert p.returncode == 0 and "Sanitizer" not in p.stderr and "runtime error" not in p.stderr, p.stderr[-4000:]
    return open(dst, "rb").read()


def expected_bytes(x, queries):
    s = oracle.compute_scales(x)
    q = oracle.quantize(x, s)
    xh = oracle.dequantize(q, s)
    ss, mx = oracle.roundtrip_error(x, xh)
    attn = oracle.attn_score_error(queries, x[0], xh[0])
    scores = oracle.scores_from_codes(queries, q[0], s[0])
    s7 = oracle.compute_scales_q(x, 7)
    q7 = oracle.quantize_q(x, s7, 7)
    s8 = oracle.compute_scales_q(x, 448)
    c8 = oracle.quantize_fp8(x, s8)
    xh8 = oracle.dequantize_fp8(c8, s8)
    enc = oracle.fp8_encode(x)
    dec = oracle.fp8_decode(enc)
    parts = [s.astype(np.float32), q.astype(np.int8), xh.astype(np.float32), np.float64(ss), np.float32(mx),
             np.float64(attn), np.asarray(scores, dtype=np.float64), s7.astype(np.float32), q7.astype(np.int8),
             c8.astype(np.uint8), xh8.astype(np.float32), enc.astype(np.uint8), dec.astype(np.float32)]
    return b"".join(np.ascontiguousarray(p).tobytes() for p in parts)


@pytest.mark.parametrize("shape,Q", [((1, 1, 1), 1), ((2, 5, 3), 2), ((3, 33, 17), 4), ((1, 64, 130), 3)],
                         ids=lambda v: str(v))
def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(driver, tmp_path, shape, Q):
    rng = np.random.default_rng(sum(shape) * 31 + Q)
    x = (rng.standard_normal(shape) * np.exp(rng.uniform(-3, 3, (shape[0], 1, shape[2])))).astype(np.float32)
    if shape[2] >= 3:
        x[:, :, 1] = 0.0                                    # zero scale
        x[0, :, 2] = np.float32(2.0 ** -140)                # subnormal entries: the scale underflows
    if shape[1] >= 5:
        x[0, 3, 0] = np.float32(3e38)                       # huge quotients before the clamp
        x[0, 4, 0] = np.float32(-3e38)
    queries = rng.standard_normal((Q, shape[2])).astype(np.float32)
    got = run_driver(driver, tmp_path, x, queries)
    want = expected_bytes(x, queries)
    assert len(got) == len(want)
    assert got == want
