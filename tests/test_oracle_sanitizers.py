"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU: builds
oracle/sanitize_driver.cpp with the oracle into one instrumented executable and runs it
(Top_K by rank over an alphabet of special values, a Lemma 1 run on dyadic inputs, the
unidirectional and the diagnostic step).  Any sanitizer report aborts the run."""
import os
import subprocess


def test_oracle_runs_clean_under_asan_and_ubsan():
    import oracle
    exe = oracle.build_sanitized()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "0 failures" in res.stdout
    assert "ERROR" not in res.stderr, res.stderr
