"""The host side of the C-ABI under AddressSanitizer and UndefinedBehaviorSanitizer (host code only: the device
code is compiled as always and never runs here).  tests/host_sanitize/driver.cpp calls every entry point with
valid and invalid arguments, the kernel launchers replaced by stubs that launch nothing."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_argument_checks_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "host_checks")
    srcs = [os.path.join(ROOT, "paper_2511_19797_amd", "csrc", "tvmattn_api.hip"),
            os.path.join(ROOT, "tests", "host_sanitize", "stubs.cpp"),
            os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp")]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    cmd = ["hipcc", "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-x", "hip",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
           *san, *srcs, "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ)
    # (the harness preloads a small library of its own in front of the sanitizer runtime; that order is harmless)
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    out = r.stdout + r.stderr
    assert r.returncode == 0 and "host checks ok" in r.stdout, out[-3000:]
    assert "runtime error" not in out and "AddressSanitizer" not in out, out[-3000:]
