"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): a small
driver calls every entry point on ragged inputs; any report ends the run with a non-zero status."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                           "-static-libasan", "-Wall", "-Wextra", "-o", exe,
                           os.path.join(ROOT, "oracle", "attn_oracle.c"), os.path.join(HERE, "oracle_sanitize_driver.c"), "-lm"])
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert r.returncode == 0, r.stdout
    assert "status 0" in r.stdout and "ERROR" not in r.stdout, r.stdout
