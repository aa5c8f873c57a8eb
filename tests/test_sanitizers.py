"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

Two small programs are built with -fsanitize=address,undefined and must run clean: the CPU
checker's C source with a driver that goes through every cache mode, and the library's host
layer (argument validation, split plan, workspace carving) with its kernel launchers stubbed
out.  GPU code is not instrumented: device-side indices are covered by the KVQ_DEBUG checks."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(exe):
    out = subprocess.run([str(exe)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                         env=ENV, timeout=300)
    assert out.returncode == 0 and " ok" in out.stdout, out.stdout[-3000:]
    assert "runtime error" not in out.stdout and "AddressSanitizer" not in out.stdout, out.stdout[-3000:]


def test_cpu_checker_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "oracle_san"
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-Wall", "-Wextra", *SAN, "-ffp-contract=off",
                           os.path.join(ROOT, "oracle", "kvq_oracle.c"),
                           os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
                           "-o", str(exe), "-lm"])
    run(exe)


def test_library_host_layer_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = tmp_path / "api_san"
    host_san = []
    for flag in SAN:
        host_san += ["-Xarch_host", flag]
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-O1", "-std=c++17",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           "-Wno-unused-command-line-argument", *host_san,
                           os.path.join(ROOT, "paper_2605_29639_amd", "csrc", "kvq_api.hip"),
                           os.path.join(ROOT, "tests", "sanitize", "api_driver.cpp"),
                           "-I", os.path.join(ROOT, "include"), "-o", str(exe)],
                          stderr=subprocess.DEVNULL)
    run(exe)
