"""CPU build of the library's host side (layout builder, argument checks, table queries) under
AddressSanitizer and UndefinedBehaviorSanitizer, driven by tests/native/host_sanitize_main.cpp:
random valid and broken batch descriptions, every table read back into an exactly sized
buffer.  The sanitizers instrument the host pass only (no device code is built or run)."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_host_side_is_clean_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "hpd_host_sanitized")
    cmd = [HIPCC, "-O1", "-g", "-std=c++17", "-x", "hip", "--offload-arch=gfx950", "--offload-host-only",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2604_26209_amd", "csrc"),
           os.path.join(ROOT, "paper_2604_26209_amd", "csrc", "hpd_host.cpp"),
           os.path.join(ROOT, "tests", "native", "host_sanitize_main.cpp"), "-o", exe]
    build = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert build.returncode == 0, build.stderr[-3000:]
    symbols = subprocess.run(["nm", exe], capture_output=True, text=True).stdout if shutil.which("nm") else "__asan_init"
    assert "__asan_init" in symbols, "the executable was not instrumented"
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "no finding" in run.stdout
    assert "ERROR: AddressSanitizer" not in run.stderr and "runtime error" not in run.stderr
