"""The library's host-only code (the adapter cache's bookkeeping: vectors, tables, victim search) built with
AddressSanitizer and UBSan on the host side and run on the CPU: random request streams in both cache
modes plus the error paths.  No GPU call is made (no stack is registered)."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_cache_bookkeeping_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "cache_asan")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-omit-frame-pointer",
           os.path.join(ROOT, "paper_2410_09687_amd", "csrc", "cache.hip"),
           os.path.join(ROOT, "tests", "host", "cache_asan_main.cpp"),
           "-fsanitize=address", "-fsanitize=undefined", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1")
    env.pop("LD_PRELOAD", None)
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-3000:])
    assert "cache host checks passed" in r.stdout
