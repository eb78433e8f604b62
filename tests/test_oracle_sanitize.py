"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only):
a small driver calls every oracle entry point on varied inputs; any report fails the run."""
import subprocess

import oracle


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = oracle.build_sanitize_driver(str(tmp_path / "sanitize_driver"))
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300,
                         env={"ASAN_OPTIONS": "detect_leaks=1:abort_on_error=0",
                              "UBSAN_OPTIONS": "print_stacktrace=1"})
    assert run.returncode == 0, run.stderr[-2000:]
    assert run.stdout.strip() == "ok"
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
