"""Host code under AddressSanitizer and UBSan (no GPU): the C oracle and kvl_plan's host logic
are driven over random batches by two small harnesses with exactly sized buffers."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "host_sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0:abort_on_error=0",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
ENV.pop("LD_PRELOAD", None)        # a preloaded library ahead of the sanitizer runtime makes it refuse to start


def _run(cmd, exe, env=ENV):
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0 and "sanitize" in (r.stderr + r.stdout).lower() and "unsupported" in (r.stderr + r.stdout).lower():
        pytest.skip("sanitizer runtime not available to this compiler")
    assert r.returncode == 0, r.stderr[-2000:]
    out = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert out.returncode == 0 and "ok" in out.stdout, (out.stdout + out.stderr)[-3000:]


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_harness")
    _run(["gcc", "-std=c99", "-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
          os.path.join(HERE, "oracle_harness.c"), os.path.join(ROOT, "oracle", "kvl_oracle.c"), "-o", exe], exe)


def test_plan_host_logic_under_asan_ubsan(tmp_path):
    hipcc = "/opt/rocm/bin/hipcc" if os.path.exists("/opt/rocm/bin/hipcc") else shutil.which("hipcc")
    if not hipcc:
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "plan_harness")
    # sanitizers on the host pass only; leak checking off because the HIP runtime keeps its own globals
    env = dict(ENV, ASAN_OPTIONS=ENV["ASAN_OPTIONS"].replace("detect_leaks=1", "detect_leaks=0"))
    _run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
          "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
          "-Wno-unused-command-line-argument",
          "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2602_21548_amd", "csrc"),
          os.path.join(ROOT, "paper_2602_21548_amd", "csrc", "kvl_plan.hip"),
          os.path.join(HERE, "plan_harness.cpp"), "-o", exe], exe, env)
