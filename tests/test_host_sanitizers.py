"""The argument checks and workspace plans of the C-ABI library under AddressSanitizer and
UndefinedBehaviorSanitizer, on the host only and without a GPU: a small C++ program
(tests/host_sanitizer_main.cpp) walks some thousand problem shapes through every size query and through every
entry point up to its last check before a launch."""
import os
import subprocess


def test_argument_checks_and_plans_are_clean_under_asan_and_ubsan(tmp_path):
    from paper_2502_00299_amd import build
    exe = build.build_host_sanitizer_check(str(tmp_path))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-4000:]
    assert "HOST SANITIZER RUN OK" in r.stdout, out[-4000:]
    assert "AddressSanitizer" not in out and "runtime error" not in out, out[-4000:]
