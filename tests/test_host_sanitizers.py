"""The library's host code (argument validation, tree analysis, workspace layout, error paths) under
AddressSanitizer and UndefinedBehaviorSanitizer: the sources are compiled with the sanitizers on the host
side only (device code is untouched) together with tests/host_sanitize_driver.cpp, which creates, queries and
destroys contexts for every benchmark tree and calls every entry point in ways that must be refused before
anything is launched.  No GPU is needed; a sanitizer report makes the driver exit non-zero."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2408_08146_amd", "csrc")
OUT = os.path.join(ROOT, "_build", "host_sanitize")


def _sources():
    from paper_2408_08146_amd.build import SOURCES
    return [os.path.join(CSRC, s) for s in SOURCES]


def test_host_code_is_clean_under_asan_and_ubsan():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    driver = os.path.join(ROOT, "tests", "host_sanitize_driver.cpp")
    deps = _sources() + [driver, os.path.join(ROOT, "include", "koala.h"), os.path.join(CSRC, "koala_internal.h")]
    if not os.path.exists(OUT) or os.path.getmtime(OUT) < max(os.path.getmtime(d) for d in deps):
        os.makedirs(os.path.dirname(OUT), exist_ok=True)
        cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xarch_device", "-O3",
               "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
               "-Xarch_host", "-fno-sanitize-recover=undefined",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC, *_sources(), "-x", "hip", driver, "-o", OUT]
        res = subprocess.run(cmd, capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-3000:]
    assert b"__asan_init" in open(OUT, "rb").read()              # the sanitizer runtime is really linked in
    env = dict(os.environ, ASAN_OPTIONS="abort_on_error=0:detect_leaks=1", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([OUT], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0, (res.stdout + res.stderr)[-3000:]
    assert "host sanitize driver: ok" in res.stdout
