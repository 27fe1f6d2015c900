"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code, CPU only): its
self-test driver runs every function on a small seeded model with exactly sized buffers and odd
dimensions; any out-of-bounds access, leak or undefined operation ends it with a non-zero status."""
import os
import subprocess


def test_oracle_selftest_is_clean_under_sanitizers(oracle, tmp_path):
    exe = oracle.build_selftest(out=str(tmp_path / "q8_oracle_selftest_san"), sanitize=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "selftest: ok" in r.stdout


def test_oracle_selftest_plain_build(oracle, tmp_path):
    exe = oracle.build_selftest(out=str(tmp_path / "q8_oracle_selftest"))
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "selftest: ok" in r.stdout, r.stdout + r.stderr
