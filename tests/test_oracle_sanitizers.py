"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only; no GPU):
oracle/sanitize_check.c calls every oracle routine on small, exactly sized heap buffers, and any
access outside an array, leak, signed overflow or bad shift aborts the run."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    src = [os.path.join(ROOT, "oracle", f) for f in ("sanitize_check.c", "aride_oracle.c")]
    # -fno-openmp: the row loop runs on the calling thread (libgomp's own allocations are not the oracle's)
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-fno-omit-frame-pointer", "-ffp-contract=off", "-Wall", "-Wextra",
           "-o", exe] + src + ["-lm"]
    subprocess.run(cmd, check=True)
    # (the sanitizer runtimes are linked statically, so the process's environment is left as it is)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip() == "ok"
