"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code, gcc).

oracle/sanitize_check.c calls every entry point of the oracle on small and awkward shapes (empty, one
token, odd N, every group size, all-zero tokens) with each buffer allocated at exactly its documented
size; any out-of-bounds access, signed overflow or invalid shift aborts the run.
"""
import subprocess

from oracle import build


def test_oracle_clean_under_asan_and_ubsan():
    exe = build.build_sanitize_check()
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                         env={"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0", "UBSAN_OPTIONS": "print_stacktrace=1"})
    assert run.returncode == 0, run.stderr[-2000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-2000:]
    assert "cases clean" in run.stdout
