"""The fp64 oracle under AddressSanitizer + UndefinedBehaviorSanitizer (host code only): the C
driver tests/sanitize_oracle.c compiles oracle/mcf_oracle.c into itself, runs every entry
point on small edge cases and checks them against a flat brute-force sum."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "sanitize_oracle")
    cmd = ["gcc", "-std=c11", "-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-Wall", "-Wextra", "-o", exe, os.path.join(HERE, "sanitize_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    env = dict(os.environ, OMP_NUM_THREADS="4", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "all cases match" in r.stdout
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr, r.stderr
