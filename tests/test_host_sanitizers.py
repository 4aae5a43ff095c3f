"""The library's host side under AddressSanitizer and UndefinedBehaviorSanitizer, without a GPU.

`csrc/pt_api.cpp` (configuration checks, arena layout, the launch sequence of prefill, decode, ragged batches and
PT-MoE) is compiled for the host with both sanitizers and linked with stand-ins for the kernel launchers
(`tests/host_check/stubs.cpp`) that launch nothing and check instead that every buffer a kernel would touch lies
inside the arenas and caller buffers of the call.  The driver walks eight model shapes through both kernel
selections, every entry point and the error paths.  A second build plants an overflow (arenas registered 512 bytes
short) and must be caught: the self-test of the checker."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HC = os.path.join(ROOT, "tests", "host_check")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build(out, extra=()):
    cmd = [HIPCC, "-x", "hip", "--offload-arch=gfx950", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2602_07306_amd", "csrc"), "-I", HC,
           *extra,
           os.path.join(ROOT, "paper_2602_07306_amd", "csrc", "pt_api.cpp"), os.path.join(HC, "stubs.cpp"),
           os.path.join(HC, "driver.cpp"), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]


def run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    return subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_host_logic_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_check")
    build(exe)
    r = run(exe)
    sys.stdout.write(r.stdout[-500:])
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "all inside their memory" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not found")
def test_the_bounds_checker_catches_a_planted_overflow(tmp_path):
    exe = str(tmp_path / "host_check_planted")
    build(exe, ["-DHC_SHRINK=512"])
    r = run(exe)
    assert r.returncode != 0
    assert "lies in no registered buffer" in r.stderr
