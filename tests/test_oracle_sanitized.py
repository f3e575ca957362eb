"""The CPU oracle under -fsanitize=address,undefined: its own C driver
(oracle/sanitize_driver.c) calls every routine over small ragged shapes with
exactly-sized buffers (a full cache, an empty suffix, selection counts above the
active positions, every sizing mode of the commit); the sanitized build must
finish without a report and print the same checksum as the plain build."""
import os
import subprocess

from oracle.build import build_sanitized


def test_every_oracle_routine_is_clean_under_asan_and_ubsan(tmp_path):
    plain, san = build_sanitized(str(tmp_path))
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0")
    a = subprocess.run([plain], capture_output=True, text=True, env=env, timeout=120)
    b = subprocess.run([san], capture_output=True, text=True, env=env, timeout=300)
    assert a.returncode == 0, a.stdout + a.stderr
    assert b.returncode == 0, b.stdout + b.stderr
    assert "runtime error" not in b.stderr and "AddressSanitizer" not in b.stderr, b.stderr
    assert a.stdout.startswith("rc=0 checksum=") and a.stdout == b.stdout, (a.stdout, b.stdout)
