"""The CPU oracle under AddressSanitizer + UndefinedBehaviorSanitizer: oracle/selftest.c calls every oracle
function on operands allocated at exactly the size the layout needs (padded pitches, batch gaps) and checks
closed forms; any access outside an operand, signed overflow or misaligned access ends the run."""
import importlib
import os
import subprocess


def test_oracle_selftest_under_sanitizers(tmp_path):
    exe = importlib.import_module("oracle.build").build_selftest(tmp_path)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "oracle selftest: ok" in r.stdout
