"""The library's host code (descriptor validation, chunk plan, workspace layout, planner) built with
AddressSanitizer and UndefinedBehaviorSanitizer and driven through every entry point that runs
without a GPU (tests/host_sanitize/driver.cpp: seeded random and boundary descriptors, random
planner inputs, output buffers with guard elements).  Any report makes the driver exit non-zero."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2301_08984_amd", "csrc")


def test_host_code_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_sanitize")
    srcs = [os.path.join(CSRC, f) for f in ("api.hip", "ffn_api.hip", "planner.hip")]
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fno-gpu-rdc",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
           "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-x", "hip", *srcs,
           os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp"),
           "-fsanitize=address", "-fsanitize=undefined", "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, (r.stdout[-2000:], r.stderr[-4000:])
    assert "all checks passed" in r.stdout
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
