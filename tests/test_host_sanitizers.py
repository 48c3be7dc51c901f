"""The library's host code (argument validation, table building, schedule planning, the walk replay,
partition, selection, group tables) under AddressSanitizer and UndefinedBehaviorSanitizer: a C++
driver (tests/host_sanitize.cpp) is compiled together with the host sources, the kernels' launchers
stubbed, and run on seeded random inputs.  No GPU is touched; the sanitizers cover host code only."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    csrc = os.path.join(ROOT, "paper_2505_13060_amd", "csrc")
    cmd = [HIPCC, "-std=c++17", "-O1", "-g", "--offload-arch=gfx950", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-x", "hip", os.path.join(ROOT, "tests", "host_sanitize.cpp"), os.path.join(ROOT, "tests", "host_hooks.cpp"),
           os.path.join(csrc, "api.hip"), os.path.join(csrc, "select.cpp"), os.path.join(csrc, "graph.cpp"),
           "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert run.returncode == 0, (run.stdout[-2000:], run.stderr[-4000:])
    assert "host_sanitize: 0 failures" in run.stdout
    shutil.rmtree(str(tmp_path), ignore_errors=True)
