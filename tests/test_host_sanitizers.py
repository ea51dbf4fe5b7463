"""The library's host code (argument checks, launch plans, workspace carving) under AddressSanitizer and
UndefinedBehaviorSanitizer: the library is built again with the sanitizers on its host side and the host boundary tests
run against that build in a child process (the sanitizer runtime has to be loaded before Python starts)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_host_boundary_tests_pass_under_asan_and_ubsan():
    from paper_2603_11564_amd import build
    try:
        runtime = build.asan_runtime()
    except RuntimeError as e:
        pytest.skip(str(e))
    lib = build.build_sanitized()
    env = dict(os.environ, DAPQ_LIBRARY=lib, LD_PRELOAD=runtime,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:halt_on_error=1",   # the interpreter itself leaks by design
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_boundary_host.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    report = r.stdout[-3000:] + r.stderr[-3000:]
    assert r.returncode == 0, report
    assert "passed" in r.stdout and "AddressSanitizer" not in report and "runtime error" not in report, report
    # the child really loaded the sanitized build
    probe = subprocess.run([sys.executable, "-c",
                            "import paper_2603_11564_amd as D; D.load_library(); print(open('/proc/self/maps').read())"],
                           cwd=ROOT, env=env, capture_output=True, text=True, timeout=120)
    assert "libdapq_san.so" in probe.stdout and "libclang_rt.asan" in probe.stdout, probe.stderr[-2000:]
