"""The host side of the C-ABI layer under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU).

The sources that hold the boundary's host logic -- argument validation, launch plans, options -- are
compiled with hipcc with the sanitizers on the host side only (device code is compiled as usual and
never runs here), and tests/sanitize_boundary_driver.c calls into the result: every entry point with
arguments that must be rejected before any HIP call, launch plans over a grid of shapes up to the
largest sizes, options at the extremes of int.  Undefined arithmetic (an index computation that
overflows, a shift too far) or a bad access ends the driver with a report."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_04719_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = "/opt/rocm/lib/llvm/bin/clang"


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANG)), reason="needs the ROCm compilers")
def test_boundary_host_code_is_clean_under_sanitizers(tmp_path):
    lib = str(tmp_path / "libkvq_host_sanitized.so")
    exe = str(tmp_path / "boundary_driver")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    srcs = [os.path.join(CSRC, f) for f in ("kvq_api.hip", "kvq_bench.hip", "kvq_absmax.hip")]
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
                    "-Wno-unused-command-line-argument"] + san + inc + ["-o", lib] + srcs, check=True,
                   stderr=subprocess.DEVNULL)
    subprocess.run([CLANG, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"] + inc +
                   ["-o", exe, os.path.join(ROOT, "tests", "sanitize_boundary_driver.c"), "-ldl"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")
    p = subprocess.run([exe, lib], env=env, capture_output=True, text=True, timeout=300)
    assert p.returncode == 0 and "runtime error" not in p.stderr and "Sanitizer" not in p.stderr, \
        (p.stdout + p.stderr)[-4000:]
    assert "launch plans:" in p.stdout and "argument validation: clean" in p.stdout
    assert "options and status strings: clean" in p.stdout
