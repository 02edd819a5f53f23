"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/sanitize_check.c drives every oracle
function on small ragged shapes and extreme values; any out-of-bounds access, signed overflow or bad shift aborts it.
No GPU."""
import os
import subprocess

import oracle


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers():
    program = oracle.build(force=True, sanitize=True)
    # verify_asan_link_order=0: the environment may preload a library of its own ahead of the sanitizer runtime
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="2")
    proc = subprocess.run([program], capture_output=True, text=True, env=env, timeout=600)
    assert proc.returncode == 0, proc.stdout + proc.stderr
    assert proc.stdout.strip() == "ok"
    assert "runtime error" not in proc.stderr and "AddressSanitizer" not in proc.stderr
