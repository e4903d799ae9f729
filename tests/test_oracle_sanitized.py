"""The CPU oracle under the address and undefined-behaviour sanitizers (host code only): a driver
calls every oracle function on small inputs that sit on the awkward sizes (no items, one item, a
list longer than the index, thresholds that keep nothing or everything, masses of equal distances);
the sanitized build must finish cleanly and print exactly what the plain build prints."""
import os
import subprocess

from oracle import icq_oracle as orc


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    plain = orc.build_sanitize_check(False, str(tmp_path))
    san = orc.build_sanitize_check(True, str(tmp_path))
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    a = subprocess.run([plain], stdout=subprocess.PIPE, stderr=subprocess.PIPE, env=env, timeout=120)
    b = subprocess.run([san], stdout=subprocess.PIPE, stderr=subprocess.PIPE, env=env, timeout=300)
    assert a.returncode == 0, a.stderr.decode()[-2000:]
    assert b.returncode == 0, "sanitizer report:\n" + b.stderr.decode()[-4000:]
    assert b"ERROR" not in b.stderr and b"runtime error" not in b.stderr, b.stderr.decode()[-4000:]
    assert a.stdout == b.stdout and a.stdout.count(b"\n") > 100
