"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): oracle/sanitize_check.c
drives every oracle function over small shapes with exactly-sized heap buffers; any out-of-bounds access, signed
overflow or misaligned access aborts the run."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_check")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-Wall", "-Wextra", "-o", exe, os.path.join(ROOT, "oracle", "sanitize_check.c"),
           os.path.join(ROOT, "oracle", "civic_oracle.c"), "-lm"]
    subprocess.check_call(cmd)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", OMP_NUM_THREADS="2")
    out = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert out.returncode == 0 and "sanitize_check OK" in out.stdout, out.stdout[-3000:]
