"""The host code of the library (partition builder, schedules, metadata) under AddressSanitizer
and UndefinedBehaviorSanitizer.  Compiling every source with the sanitizers takes about a minute
and a half, so the test runs only when GNNMI_SANITIZE=1 is set:

    GNNMI_SANITIZE=1 python -m pytest tests/test_host_sanitizers.py -q
"""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(os.environ.get("GNNMI_SANITIZE") != "1", reason="set GNNMI_SANITIZE=1 (90 s build)")
def test_partition_builder_is_clean_under_sanitizers(tmp_path):
    from paper_2605_11517_amd.build import CSRC, HIPCC, INCLUDE, SOURCES
    exe = str(tmp_path / "host_sanitizers")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-I", INCLUDE, "-I", CSRC,
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer", "-Wno-unused-command-line-argument",
           os.path.join(ROOT, "tests", "host_sanitizers.cpp")]
    cmd += [os.path.join(CSRC, s) for s in SOURCES] + ["-o", exe, "-lpthread"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=900)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "failures: 0" in r.stdout
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
