"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU): oracle.c and its
driver (oracle/sanitize_main.c) are compiled with -fsanitize=address,undefined and run over small
seeded fp32 and bf16 models, ragged windows, trees, the greedy rule and the degenerate cases.  The
checker that every parity claim rests on must itself be free of out-of-bounds accesses, reads of
uninitialised or freed memory and undefined arithmetic."""
import os
import subprocess

import oracle


def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = oracle.build_sanitized(str(tmp_path))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    out = r.stdout + r.stderr
    assert r.returncode == 0, out[-4000:]
    assert "runtime error" not in out and "AddressSanitizer" not in out and "LeakSanitizer" not in out, out[-4000:]
    assert "0 failed checks" in out
