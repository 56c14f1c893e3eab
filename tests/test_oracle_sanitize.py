"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): oracle/sanitize_check.c calls
every entry point of oracle/eck_oracle.c on small, exactly sized heap buffers (ragged sizes included); any access
outside a buffer, signed overflow, bad shift or misaligned access aborts it with a report."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    subprocess.check_call(["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-fno-omit-frame-pointer", "-ffp-contract=off", "-o", exe, "sanitize_check.c", "-lm"],
                          cwd=os.path.join(ROOT, "oracle"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    sys.stdout.write(res.stdout[-4000:])
    assert res.returncode == 0, res.stdout[-4000:]
    assert "sanitize_check ok" in res.stdout and "runtime error" not in res.stdout
