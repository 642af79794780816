"""The sanitizer leg (opt-in: `pytest tests/test_sanitizers.py --sanitizers`, CPU only, a few minutes).

The oracle (plain C) is rebuilt with gcc's AddressSanitizer and UndefinedBehaviorSanitizer and every CPU test of it
runs again on that build; the objects of the HIP library are rebuilt with the two sanitizers in their HOST code (the GPU
side is the ordinary one: device sanitizers are not used) and linked with tests/host_abi_check.c, a C program that walks
the host-only entry points (token schedule, workspace size, saved-activation report, configuration checks, error
paths, tile-shape list).  Each runs in a child process; a report from either sanitizer fails the test."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _wanted(request):
    if not request.config.getoption("--sanitizers"):
        pytest.skip("sanitizer leg: run with --sanitizers")


def test_oracle_under_asan_and_ubsan(request, tmp_path):
    _wanted(request)
    from oracle.binding import build_oracle_sanitized
    build_oracle_sanitized(str(tmp_path))
    pre = [subprocess.run(["gcc", f"-print-file-name={n}"], capture_output=True, text=True).stdout.strip()
           for n in ("libasan.so", "libubsan.so")]
    env = dict(os.environ)
    env["LD_PRELOAD"] = " ".join(filter(None, [env.get("LD_PRELOAD", "")] + pre))
    # python itself is not instrumented: its own leaks are not ours
    env["ASAN_OPTIONS"] = "detect_leaks=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                        "--bsr-libs", str(tmp_path), "tests/test_oracle_layers.py", "tests/test_oracle_moe.py",
                        "tests/test_oracle_step.py"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert r.returncode == 0 and " passed" in out, out[-4000:]


def test_host_code_of_the_hip_library_under_asan_and_ubsan(request, tmp_path):
    _wanted(request)
    from paper_2405_10951_amd import build
    exe = build.build_sanitized_program(os.path.join(ROOT, "tests", "host_abi_check.c"), str(tmp_path))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:exitcode=99", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1:exitcode=98")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    out = r.stdout + r.stderr
    assert "AddressSanitizer" not in out and "runtime error:" not in out, out[-4000:]
    assert r.returncode == 0 and "all checks passed" in out, out[-4000:]
