"""The C oracle under gcc's address and undefined-behaviour sanitizers (CPU only): a driver calls every exported
function on small edge-case shapes with exactly sized arrays; any out-of-bounds access, use of an uninitialised
index, signed overflow or misaligned access aborts the run with a report."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-static-libasan", "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "oracle", "flare_oracle.c"), os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"),
           "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    sys.stdout.write(run.stdout)
    sys.stderr.write(run.stderr)
    assert run.returncode == 0, run.stderr[-2000:]
    assert run.stdout.strip() == "ok"
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr
